// Host-side task-graph compiler (paper Section 4.1 and the launch-mode labelling of Section 5.2).
//
//   K1  operator list of one decode step (fusion flags applied here)
//   K2  operator decomposition: each operator's OUTPUT tensor is cut into disjoint tiles, one
//       task per tile (Section 4.1 "operator decomposition")
//   K3  dependency analysis: task t1 -> t2 iff t1's output region overlaps a region t2 reads
//       (Section 4.1 "dependency analysis"), evaluated with interval arithmetic on tile bounds
//   K4  event fusion: successor-set (Def. 4.1) then predecessor-set (Def. 4.2)
//   K5  normalization: at most one dependent and one triggering event per task (Fig. 5)
//   K6  linearization: Algorithm 1, events store [first, last) into the task list
//   K7  JIT / AOT labels per operator and round-robin pre-enqueue of AOT tasks (Section 5.2)
//
// Integer-only; runs once per mpk_compile.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <map>
#include <numeric>
#include <unordered_map>

#include "mpk_internal.h"

namespace mpk {

static thread_local char g_err[512] = "";
void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
const char* last_error() { return g_err; }

// ------------------------------------------------------------------ tiling helpers
// n units in k contiguous tiles: the first n % k tiles hold ceil(n / k) units, the rest floor.
static inline uint32_t tile_begin(uint32_t n, uint32_t k, uint32_t i) {
  uint32_t q = n / k, r = n % k;
  return i * q + std::min(i, r);
}
static inline uint32_t tile_of(uint32_t n, uint32_t k, uint32_t u) {
  uint32_t q = n / k, r = n % k;
  uint32_t big = r * (q + 1);
  if (u < big) return u / (q + 1);
  return r + (u - big) / q;   // q > 0 here because k <= n is enforced at decomposition
}

// Column tiles of an operator, in units.  Usually one even split; an operator with seg_tiles
// (the QKV projection) is split twice: into segments of align_unit units (heads), and every
// segment evenly into seg_tiles tiles, so that no tile straddles a head whatever its size.
static inline uint32_t col_tile_begin(const HostOp& op, uint32_t ic) {
  const uint32_t nu = op.cols / op.unit;
  if (!op.col_begin.empty()) return op.col_begin[std::min<size_t>(ic, op.col_begin.size() - 1)];
  if (!op.seg_tiles) return tile_begin(nu, op.tc, ic);
  if (ic >= op.tc) return nu;
  return ic / op.seg_tiles * op.align_unit + tile_begin(op.align_unit, op.seg_tiles, ic % op.seg_tiles);
}
static inline uint32_t col_tile_of(const HostOp& op, uint32_t u) {
  const uint32_t nu = op.cols / op.unit;
  if (!op.col_begin.empty())   // the tile whose [begin, next begin) holds u
    return (uint32_t)(std::upper_bound(op.col_begin.begin(), op.col_begin.end(), u) - op.col_begin.begin()) - 1u;
  if (!op.seg_tiles) return tile_of(nu, op.tc, u);
  return u / op.align_unit * op.seg_tiles + tile_of(op.align_unit, op.seg_tiles, u % op.align_unit);
}
static inline uint32_t col_tile_max_units(const HostOp& op) {
  const uint32_t nu = op.cols / op.unit;
  if (!op.col_begin.empty()) {
    uint32_t m = 0;
    for (size_t i = 0; i + 1 < op.col_begin.size(); ++i) m = std::max(m, op.col_begin[i + 1] - op.col_begin[i]);
    return m;
  }
  if (!op.seg_tiles) return (nu + op.tc - 1) / op.tc;
  return (op.align_unit + op.seg_tiles - 1) / op.seg_tiles;
}

struct Rect {
  int tensor;
  uint32_t b0, b1, c0, c1;
};

// ------------------------------------------------------------------ generic graph passes
struct Ev {
  std::vector<uint32_t> in, out;   // sorted task ids
};

struct VecHash {
  size_t operator()(const std::vector<uint32_t>& v) const {
    uint64_t h = 0x9E3779B97F4A7C15ull ^ v.size();
    for (uint32_t x : v) {
      h ^= x + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
    }
    return (size_t)h;
  }
};

static void sort_unique(std::vector<uint32_t>& v) {
  std::sort(v.begin(), v.end());
  v.erase(std::unique(v.begin(), v.end()), v.end());
}

// Def. 4.1: events with equal OutTasks become one event whose InTasks is the union.
static std::vector<Ev> successor_set_fusion(std::vector<Ev>& evs) {
  std::unordered_map<std::vector<uint32_t>, size_t, VecHash> by;
  std::vector<Ev> out;
  for (auto& e : evs) {
    auto it = by.find(e.out);
    if (it == by.end()) {
      by.emplace(e.out, out.size());
      out.push_back(std::move(e));
    } else {
      auto& dst = out[it->second].in;
      dst.insert(dst.end(), e.in.begin(), e.in.end());
    }
  }
  for (auto& e : out) sort_unique(e.in);
  return out;
}

// Def. 4.2: events with equal InTasks become one event whose OutTasks is the union.
static std::vector<Ev> predecessor_set_fusion(std::vector<Ev>& evs) {
  std::unordered_map<std::vector<uint32_t>, size_t, VecHash> by;
  std::vector<Ev> out;
  for (auto& e : evs) {
    auto it = by.find(e.in);
    if (it == by.end()) {
      by.emplace(e.in, out.size());
      out.push_back(std::move(e));
    } else {
      auto& dst = out[it->second].out;
      dst.insert(dst.end(), e.out.begin(), e.out.end());
    }
  }
  for (auto& e : out) sort_unique(e.out);
  return out;
}

// Fig. 5 rewrites.  Tasks that trigger the same set of k > 1 events share one new event and k
// dummy tasks (one per original event); likewise for tasks that depend on the same set of k > 1
// events.  Dummy ids start at *n_tasks and *n_tasks is advanced.
static void normalize(std::vector<Ev>& evs, uint32_t* n_tasks) {
  for (int pass = 0; pass < 2; ++pass) {
    // pass 0: fan-out (lists = events a task triggers); pass 1: fan-in (events it depends on)
    std::vector<std::vector<uint32_t>> lists(*n_tasks);
    for (uint32_t ei = 0; ei < evs.size(); ++ei)
      for (uint32_t t : (pass == 0 ? evs[ei].in : evs[ei].out)) lists[t].push_back(ei);
    std::map<std::vector<uint32_t>, std::vector<uint32_t>> groups;   // ordered: deterministic
    for (uint32_t t = 0; t < lists.size(); ++t)
      if (lists[t].size() > 1) groups[lists[t]].push_back(t);
    for (auto& kv : groups) {
      const std::vector<uint32_t>& es = kv.first;
      const std::vector<uint32_t>& ts = kv.second;   // sorted by construction
      Ev fresh;
      std::vector<uint32_t> dummies;
      for (uint32_t ei : es) {
        uint32_t dmy = (*n_tasks)++;
        dummies.push_back(dmy);
        auto& side = (pass == 0 ? evs[ei].in : evs[ei].out);
        std::vector<uint32_t> kept;
        std::set_difference(side.begin(), side.end(), ts.begin(), ts.end(),
                            std::back_inserter(kept));
        kept.push_back(dmy);   // dummy ids exceed all earlier ids: stays sorted
        side.swap(kept);
      }
      if (pass == 0) {
        fresh.in = ts;
        fresh.out = dummies;
      } else {
        fresh.in = dummies;
        fresh.out = ts;
      }
      evs.push_back(std::move(fresh));
    }
  }
}

struct PassInput {
  uint32_t n_real = 0;
  std::vector<std::vector<uint32_t>> prod;   // per task: sorted direct producers
  std::vector<uint32_t> op_of;               // per real task: operator index (or 0)
  std::vector<uint32_t> op_jit;              // per operator: 1 = JIT
  std::vector<uint32_t> tile_of_task;        // per real task
  std::vector<std::vector<uint32_t>> prod_before;   // transitive reduction: sets before pruning
  std::vector<uint64_t> scratch_anc;
};

static mpk_status run_passes(PassInput& in, const mpk_compile_options& opt, HostGraph& g) {
  const uint32_t n_real = in.n_real;
  g.n_real = n_real;
  // --- K3 result -> one event per consumer.  Every pair event (t1, t2) has OutTasks = {t2}, so
  // grouping the pairs by consumer IS successor-set fusion applied to the pair events; the
  // function is still run so that arbitrary inputs take the same path.
  uint64_t n_pairs = 0;
  std::vector<Ev> evs;
  for (uint32_t t = 0; t < n_real; ++t) {
    if (in.prod[t].empty()) continue;
    n_pairs += in.prod[t].size();
    Ev e;
    e.in = in.prod[t];
    e.out = {t};
    evs.push_back(std::move(e));
  }
  g.stats.n_pair_deps = n_pairs;
  evs = successor_set_fusion(evs);
  evs = predecessor_set_fusion(evs);
  g.stats.n_events_fused = (uint32_t)evs.size();
  uint64_t succ_entries = 0;
  for (auto& e : evs) succ_entries += e.out.size();

  // --- K5
  uint32_t n_tasks = n_real;
  normalize(evs, &n_tasks);
  g.stats.n_dummy_tasks = n_tasks - n_real;

  // terminal event: tasks that trigger nothing notify it, its range is empty
  std::vector<int32_t> dep_of(n_tasks, -1), trig_of(n_tasks, -1);
  for (uint32_t ei = 0; ei < evs.size(); ++ei) {
    for (uint32_t t : evs[ei].out) {
      if (dep_of[t] != -1) { set_error("normalization left task %u with two dependent events", t); return MPK_ERR_INTERNAL; }
      dep_of[t] = (int32_t)ei;
    }
    for (uint32_t t : evs[ei].in) {
      if (trig_of[t] != -1) { set_error("normalization left task %u with two triggering events", t); return MPK_ERR_INTERNAL; }
      trig_of[t] = (int32_t)ei;
    }
  }
  {
    Ev term;
    for (uint32_t t = 0; t < n_tasks; ++t)
      if (trig_of[t] == -1) term.in.push_back(t);
    for (uint32_t t : term.in) trig_of[t] = (int32_t)evs.size();
    evs.push_back(std::move(term));
  }
  const uint32_t term_old = (uint32_t)evs.size() - 1;

  // --- K6: Algorithm 1.  Event ids are renumbered in dequeue order; the start event is id 0.
  std::vector<std::vector<uint32_t>> members(evs.size());
  std::vector<uint32_t> sources;
  for (uint32_t t = 0; t < n_tasks; ++t) {
    if (dep_of[t] < 0) sources.push_back(t);
    else members[dep_of[t]].push_back(t);   // ascending task id: (op, tile) order, dummies last
  }
  std::vector<uint32_t> remaining(evs.size());
  for (uint32_t ei = 0; ei < evs.size(); ++ei) remaining[ei] = (uint32_t)evs[ei].in.size();
  std::vector<int32_t> new_id(evs.size(), -1);
  std::vector<uint32_t> order;          // old task ids in linearized order
  std::vector<uint32_t> pos(n_tasks, UINT32_MAX);
  std::vector<EventDesc> events;
  std::deque<int32_t> q;
  q.push_back(-1);   // start event
  while (!q.empty()) {
    int32_t e = q.front();
    q.pop_front();
    const std::vector<uint32_t>& mem = (e < 0) ? sources : members[e];
    EventDesc d{};
    d.required = (e < 0) ? 0u : (uint32_t)evs[e].in.size();
    d.first = (uint32_t)order.size();
    if (e >= 0) new_id[e] = (int32_t)events.size();
    for (uint32_t t : mem) {
      pos[t] = (uint32_t)order.size();
      order.push_back(t);
      int32_t e2 = trig_of[t];
      if (e2 >= 0 && --remaining[e2] == 0) q.push_back(e2);
    }
    d.last = (uint32_t)order.size();
    events.push_back(d);
  }
  if (order.size() != n_tasks) { set_error("linearization placed %zu of %u tasks (cycle?)", order.size(), n_tasks); return MPK_ERR_INTERNAL; }
  for (uint32_t ei = 0; ei < evs.size(); ++ei)
    if (new_id[ei] < 0) { set_error("event %u never activated during linearization", ei); return MPK_ERR_INTERNAL; }
  g.start_event = 0;
  g.terminal_event = (uint32_t)new_id[term_old];

  // --- K7: launch modes.  A dummy task is AOT.  An event that launches at least one JIT task is
  // handled by a scheduler.
  const bool have_sched = opt.n_sched_wgs > 0 && !opt.force_aot;
  g.tasks.resize(n_tasks);
  uint32_t n_jit = 0;
  for (uint32_t i = 0; i < n_tasks; ++i) {
    uint32_t t = order[i];
    HostTask& ht = g.tasks[i];
    bool real = t < n_real;
    ht.op = real ? in.op_of[t] : MPK_TASK_DUMMY_OP;
    ht.tile = real ? in.tile_of_task[t] : (t - n_real);
    ht.dep_event = dep_of[t] < 0 ? 0 : new_id[dep_of[t]];   // sources depend on the start event
    ht.trig_event = new_id[trig_of[t]];
    ht.jit = (real && have_sched && !in.op_jit.empty() && in.op_jit[in.op_of[t]]) ? 1u : 0u;
    ht.worker = -1;
    n_jit += ht.jit;
  }
  for (auto& e : events) {
    e.flags = 0;
    for (uint32_t i = e.first; i < e.last; ++i)
      if (g.tasks[i].jit) e.flags |= 1u;
  }
  g.events = events;
  const uint32_t W = opt.n_workers;
  std::vector<std::vector<uint32_t>> queues(W);
  uint32_t cursor = 0;
  for (uint32_t i = 0; i < n_tasks; ++i) {
    if (g.tasks[i].jit) continue;
    g.tasks[i].worker = (int32_t)(cursor % W);
    queues[cursor % W].push_back(i);
    ++cursor;
  }
  g.aot_off.assign(W + 1, 0);
  g.aot.clear();
  for (uint32_t w = 0; w < W; ++w) {
    g.aot_off[w] = (uint32_t)g.aot.size();
    g.aot.insert(g.aot.end(), queues[w].begin(), queues[w].end());
  }
  g.aot_off[W] = (uint32_t)g.aot.size();

  // Wide events whose producers all have a fixed worker (AOT) count arrivals per worker group.
  g.n_hier_events = 0;
  {
    std::vector<std::vector<uint32_t>> sub(g.events.size(), std::vector<uint32_t>(8, 0));
    std::vector<uint8_t> has_jit_producer(g.events.size(), 0);
    for (uint32_t i = 0; i < n_tasks; ++i) {
      int32_t e = g.tasks[i].trig_event;
      if (g.tasks[i].jit) has_jit_producer[e] = 1;
      else sub[e][(uint32_t)g.tasks[i].worker & 7u]++;
    }
    for (size_t e = 0; e < g.events.size(); ++e) {
      EventDesc& ev = g.events[e];
      if (ev.required < kHierMinRequired || has_jit_producer[e]) continue;
      ev.flags |= EV_HIER;
      ev.hier_slot = g.n_hier_events++;
      ev.n_groups = 0;
      for (int k = 0; k < 8; ++k) {
        ev.sub_required[k] = sub[e][k];
        ev.n_groups += sub[e][k] ? 1u : 0u;
      }
    }
  }

  g.stats.n_tasks = n_tasks;
  g.stats.n_events = (uint32_t)events.size();
  g.stats.n_jit_tasks = n_jit;
  g.stats.n_aot_tasks = n_tasks - n_jit;
  g.stats.successor_bytes_unlinearized = 4 * (succ_entries + g.stats.n_dummy_tasks);
  g.stats.successor_bytes_linearized = 8ull * events.size();
  g.stats.n_workers = W;
  g.stats.n_sched_wgs = opt.n_sched_wgs;
  g.stats.task_desc_bytes = sizeof(TaskDesc);
  return MPK_OK;
}

// ------------------------------------------------------------------ transitive reduction
// Drops a pair (p, t) when p is already an ancestor of another direct producer of t.  Ancestor
// sets are bitsets over a sliding window of operators: an implied path from p to t only visits
// operators between op(p) and op(t), and no pair spans more than `max_span` operators.
static uint64_t transitive_reduction(PassInput& in, const std::vector<HostOp>& ops) {
  const uint32_t n = in.n_real;
  uint32_t max_span = 1;
  for (uint32_t t = 0; t < n; ++t)
    for (uint32_t p : in.prod[t]) max_span = std::max(max_span, in.op_of[t] - in.op_of[p]);
  auto window_base = [&](uint32_t op) {
    uint32_t lo = op > max_span ? op - max_span : 0;
    return ops[lo].task_base;
  };
  std::vector<std::vector<uint64_t>> anc(n);   // bit i = task (window_base(op(t)) + i)
  in.prod_before.assign(n, {});
  uint64_t removed = 0;
  uint32_t free_below = 0;
  for (uint32_t t = 0; t < n; ++t) {
    uint32_t op = in.op_of[t];
    uint32_t base = window_base(op);
    // release ancestor sets that can no longer be referenced
    while (free_below < base) {
      std::vector<uint64_t>().swap(anc[free_below]);
      ++free_below;
    }
    uint32_t nbits = t - base;
    std::vector<uint64_t> u((nbits + 63) / 64 + 1, 0);   // union of producers' ancestors
    auto& P = in.prod[t];
    if (t > 0 && in.op_of[t - 1] == op && in.prod_before[t - 1] == P) {
      u = anc[t - 1];   // same producer set as the previous tile: same ancestors
      u.resize((nbits + 63) / 64 + 1, 0);
    } else {
      for (uint32_t p : P) {
        // anc[p] bit j is task pb + j with pb <= base: shift right by s = base - pb
        uint32_t s = base - window_base(in.op_of[p]);
        const auto& a = anc[p];
        size_t ws = s >> 6, bs = s & 63;
        for (size_t k = 0; k < u.size(); ++k) {
          uint64_t lo = (k + ws < a.size()) ? a[k + ws] : 0;
          uint64_t hi = (k + ws + 1 < a.size()) ? a[k + ws + 1] : 0;
          u[k] |= bs ? ((lo >> bs) | (hi << (64 - bs))) : lo;
        }
        u[(p - base) >> 6] |= 1ull << ((p - base) & 63);
      }
      // u now holds P and all ancestors; strip P's own bits unless implied by another producer
      std::vector<uint64_t> self(u.size(), 0);
      for (uint32_t p : P) {
        uint32_t s = base - window_base(in.op_of[p]);
        const auto& a = anc[p];
        size_t ws = s >> 6, bs = s & 63;
        for (size_t k = 0; k < self.size(); ++k) {
          uint64_t lo = (k + ws < a.size()) ? a[k + ws] : 0;
          uint64_t hi = (k + ws + 1 < a.size()) ? a[k + ws + 1] : 0;
          self[k] |= bs ? ((lo >> bs) | (hi << (64 - bs))) : lo;
        }
      }
      in.scratch_anc.swap(self);   // ancestors only (without P itself)
    }
    const std::vector<uint64_t>& only_anc = in.scratch_anc;
    std::vector<uint32_t> kept;
    for (uint32_t p : P) {
      bool implied = ((p - base) >> 6) < only_anc.size() &&
                     ((only_anc[(p - base) >> 6] >> ((p - base) & 63)) & 1);
      if (implied) ++removed;
      else kept.push_back(p);
    }
    in.prod_before[t] = P;
    P.swap(kept);
    anc[t].swap(u);
  }
  return removed;
}

// ------------------------------------------------------------------ K1: operator list
struct Builder {
  const mpk_model_config& c;
  const mpk_compile_options& o;
  HostGraph& g;
  int new_tensor(uint32_t rows, uint32_t cols, bool external = false) {
    HostTensor t{rows, cols, external ? SIZE_MAX : g.arena_floats};
    if (!external) g.arena_floats += ((size_t)rows * cols + 63) / 64 * 64;
    g.tensors.push_back(t);
    return (int)g.tensors.size() - 1;
  }
  HostOp& add(uint32_t kind, int layer, const char* name, int out, uint32_t unit, int in1,
              int in2 = -1) {
    HostOp op{};
    op.kind = kind;
    op.layer = layer;
    op.name = (layer >= 0 ? "L" + std::to_string(layer) + "." : std::string()) + name;
    op.out_tensor = out;
    op.rows = g.tensors[out].rows;
    op.cols = g.tensors[out].cols;
    op.unit = unit;
    op.in_tensor = in1;
    op.in2_tensor = in2;
    g.ops.push_back(op);
    return g.ops.back();
  }
};

static mpk_status build_ops(const mpk_model_config& c, const mpk_weight_ptrs* w,
                            const mpk_compile_options& o, uint32_t C, HostGraph& g) {
  Builder b{c, o, g};
  const uint32_t B = c.batch, H = c.hidden, d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads;
  const uint32_t F = c.ffn, V = c.vocab, grp = nq / nkv, QKV = (nq + 2 * nkv) * d;
  const uint32_t f = o.fusion;
  mpk_layer_weights none{};
  int x = b.new_tensor(B, H);
  // When the residual stream comes out of a split-K operator, dependencies go through that
  // operator's partial tensor x_dep ([B][x_parts x H]) while bodies load x.
  int x_dep = -1;
  uint32_t x_parts = 0;
  auto reads_x = [&](HostOp& op, bool second) {   // op reads the residual stream as in (or in2)
    if (x_dep < 0) return;
    if (second) { op.in2_tensor = x_dep; op.body_in2_tensor = x; op.in2_kparts = x_parts; }
    else { op.in_tensor = x_dep; op.body_in_tensor = x; op.in_kparts = x_parts; }
  };
  // Serving (Section 6.1): ONE task on the start event prepares the iteration -- it retires and
  // admits requests and updates the paged-cache metadata -- and writes one metadata element per
  // batch slot; slot b's embedding reads element b, so the whole iteration is downstream of it.
  int slots = -1;
  if (o.serving) {
    slots = b.new_tensor(B, 1);
    b.add(MPK_OP_SERVE, -1, "serve", slots, 1, -1);
  }
  {
    HostOp& op = b.add(MPK_OP_EMBED, -1, "embed", x, H, slots);
    op.w = w ? w->embed : nullptr;
    op.K = H;
  }
  for (uint32_t l = 0; l < c.n_layers; ++l) {
    const mpk_layer_weights& lw = (w && w->layers) ? w->layers[l] : none;
    int qkv_in = x;
    if (!(f & MPK_FUSE_NORM)) {
      int xn = b.new_tensor(B, H);
      HostOp& op = b.add(MPK_OP_RMSNORM, l, "attn_norm", xn, H, x);
      op.w2 = lw.attn_norm; op.f0 = c.rms_eps; op.K = H;
      qkv_in = xn;
    }
    int qkv = b.new_tensor(B, QKV);
    {
      HostOp& op = b.add(MPK_OP_LINEAR, l, "qkv", qkv, 1, qkv_in);
      op.w = lw.wqkv; op.K = H; op.align_unit = d;
      if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = lw.attn_norm; op.f0 = c.rms_eps; reads_x(op, false); }
    }
    int qsrc = qkv;
    if (!(f & MPK_FUSE_ROPE)) {
      int rk = b.new_tensor(B, QKV);
      HostOp& op = b.add(MPK_OP_ROPE, l, "rope", rk, d, qkv);
      op.f1 = c.rope_theta; op.p0 = l;
      if (c.flags & MPK_MODEL_QK_NORM) { op.flags |= TF_QK_NORM; op.w = lw.q_norm; op.w2 = lw.k_norm; op.f0 = c.rms_eps; }
      qsrc = rk;
    }
    int part = b.new_tensor(B, nkv * C * grp * (d + 2));
    {
      HostOp& op = b.add(MPK_OP_ATTN_PARTIAL, l, "attn_partial", part, grp * (d + 2), qsrc);
      op.p0 = l; op.p1 = C; op.f1 = c.rope_theta;
      if (o.kv_page_size) op.flags |= TF_KV_PAGED;
      if (f & MPK_FUSE_ROPE) {
        op.flags |= TF_ROPE_FUSED;
        if (c.flags & MPK_MODEL_QK_NORM) { op.flags |= TF_QK_NORM; op.w = lw.q_norm; op.w2 = lw.k_norm; op.f0 = c.rms_eps; }
      }
    }
    int osrc = part, o_body = -1;
    uint32_t oK = nq * d;
    if (!(f & MPK_FUSE_MERGE)) {
      int ot = b.new_tensor(B, nq * d);
      HostOp& op = b.add(MPK_OP_ATTN_MERGE, l, "attn_merge", ot, d, part);
      op.p1 = C;
      osrc = ot;
    } else {
      // The chunk task that finishes last for a (sequence, KV head) merges the partials into o;
      // the O projection depends on the partial buffer (all chunk tasks) and loads o.
      o_body = b.new_tensor(B, nq * d);
      HostOp& at = g.ops.back();
      at.flags |= TF_ATTN_MERGE;
      at.side_out_tensor = o_body;
      at.p2 = l * B * nkv;   // first arrival counter of this layer
      if (B > 1 && !o.no_attn_balance) at.flags |= TF_ATTN_BALANCE;
    }
    int x1 = b.new_tensor(B, H);
    if (f & MPK_FUSE_RESID) {
      HostOp& op = b.add(MPK_OP_LINEAR, l, "o_proj", x1, 1, osrc, x);
      op.w = lw.wo; op.K = oK; op.flags |= TF_EPI_RESID;
      op.body_in_tensor = o_body;
      reads_x(op, true);
    } else {
      int a = b.new_tensor(B, H);
      HostOp& op = b.add(MPK_OP_LINEAR, l, "o_proj", a, 1, osrc);
      op.w = lw.wo; op.K = oK;
      op.body_in_tensor = o_body;
      b.add(MPK_OP_ADD, l, "resid1", x1, 1, x, a);
    }
    int gin = x1;
    if (!(f & MPK_FUSE_NORM)) {
      int xn2 = b.new_tensor(B, H);
      HostOp& op = b.add(MPK_OP_RMSNORM, l, "mlp_norm", xn2, H, x1);
      op.w2 = lw.mlp_norm; op.f0 = c.rms_eps; op.K = H;
      gin = xn2;
    }
    if (c.n_experts) {
      // Mixture-of-experts block (Section 6.4): router, route (softmax + top-k -> meta-tensor),
      // the experts' gate/up stage, their down stage, combine.  An expert stage is cut into a
      // fixed number of expert tasks at compile time; which rows of which expert a task works on
      // is refined at run time from the meta-tensor, so for the dependency analysis a stage's
      // output is one element per task and every consumer reads all of them.
      const uint32_t E = c.n_experts, TK = c.top_k, Fe = c.expert_ffn, P = B * TK;
      const uint32_t NT = o.tiles_moe ? o.tiles_moe : o.n_workers;
      int rl = b.new_tensor(B, E);
      {
        HostOp& op = b.add(MPK_OP_LINEAR, l, "router", rl, 1, gin);
        op.w = lw.router; op.K = H;
        if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = lw.mlp_norm; op.f0 = c.rms_eps; }
      }
      int meta = b.new_tensor(1, 1), meta_data = b.new_tensor(1, moe_meta_words(E, P));
      g.moe_meta_offset.push_back(g.tensors[meta_data].offset);
      {
        HostOp& op = b.add(MPK_OP_ROUTER, l, "route", meta, 1, rl);
        op.data_in = rl; op.data_out = meta_data;
        op.p0 = E; op.p1 = TK; op.p2 = B; op.K = E;
      }
      int eh = b.new_tensor(1, NT), hbuf = b.new_tensor(P, Fe);
      {
        HostOp& op = b.add(MPK_OP_EXPERT, l, "expert_gate_up", eh, 1, meta, gin);
        op.data_in = gin; op.data_in2 = meta_data; op.data_out = hbuf;
        op.w = lw.expert_wgu; op.K = H; op.flags |= TF_GATEUP;
        op.p0 = Fe; op.p1 = NT; op.p2 = 2 * Fe; op.p3 = E | (TK << 16);
        if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = lw.mlp_norm; op.f0 = c.rms_eps; }
      }
      int ey = b.new_tensor(1, NT), ybuf = b.new_tensor(P, H);
      {
        HostOp& op = b.add(MPK_OP_EXPERT, l, "expert_down", ey, 1, meta, eh);
        op.data_in = hbuf; op.data_in2 = meta_data; op.data_out = ybuf;
        op.w = lw.expert_wd; op.K = Fe;
        op.p0 = 0; op.p1 = NT; op.p2 = H; op.p3 = E | (TK << 16);
      }
      int xo = b.new_tensor(B, H);
      {
        HostOp& op = b.add(MPK_OP_COMBINE, l, "combine", xo, 1, x1, ey);
        op.in3_tensor = meta;
        op.data_in = ybuf; op.data_in2 = x1; op.data_aux = meta_data; op.data_out = xo;
        op.p0 = E; op.p1 = TK; op.K = H;
      }
      x = xo;
      continue;
    }
    int h = b.new_tensor(B, F);
    if (f & MPK_FUSE_SWIGLU) {
      HostOp& op = b.add(MPK_OP_GATEUP, l, "gate_up", h, 1, gin);
      op.w = lw.wgu; op.K = H; op.flags |= TF_GATEUP; op.p0 = F;
      if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = lw.mlp_norm; op.f0 = c.rms_eps; }
    } else {
      int gu = b.new_tensor(B, 2 * F);
      HostOp& op = b.add(MPK_OP_LINEAR, l, "gate_up", gu, 1, gin);
      op.w = lw.wgu; op.K = H;
      if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = lw.mlp_norm; op.f0 = c.rms_eps; }
      HostOp& sw = b.add(MPK_OP_SWIGLU, l, "swiglu", h, 1, gu);
      sw.p0 = F;
    }
    // Batch > 4 and an input several staging tiles long: every task would re-read the whole
    // input (as many bytes as its weights).  Split the input range over `parts` tasks per row
    // block instead; the last task of a row block to arrive adds the parts (in order) and the
    // residual.  Only in the fully fused operator list, where the readers of the result are
    // linear operators.
    uint32_t parts = 1;
    if (B > 4 && (f & MPK_FUSE_RESID) && (f & MPK_FUSE_NORM) && !o.tiles_linear) {
      const uint32_t kt = B <= 8 ? 2048u : 1024u, W = o.n_workers;
      for (uint32_t kp = 4; kp >= 2 && parts == 1; kp >>= 1) {
        const uint32_t per = (uint64_t)kp * H % W == 0 ? kp * H / W : 0;   // rows per task
        if (F % (kp * 64) == 0 && F / kp >= kt && F >= 3 * kt && per >= 16 && per % 16 == 0 && per <= 512 && H % per == 0) parts = kp;
      }
    }
    if (parts > 1) {
      int dpart = b.new_tensor(B, parts * H);
      int xo = b.new_tensor(B, H);
      HostOp& op = b.add(MPK_OP_LINEAR, l, "down", dpart, 1, h, x1);
      op.w = lw.wd; op.K = F; op.flags |= TF_EPI_RESID | TF_SPLITK;
      op.p0 = parts; op.p1 = H; op.p2 = g.n_splitk_counters;
      op.side_out_tensor = xo;
      g.n_splitk_counters += o.n_workers / parts;   // one arrival counter per row block
      x = xo; x_dep = dpart; x_parts = parts;
      continue;
    }
    x_dep = -1; x_parts = 0;
    int xo = b.new_tensor(B, H);
    if (f & MPK_FUSE_RESID) {
      HostOp& op = b.add(MPK_OP_LINEAR, l, "down", xo, 1, h, x1);
      op.w = lw.wd; op.K = F; op.flags |= TF_EPI_RESID;
    } else {
      int m = b.new_tensor(B, H);
      HostOp& op = b.add(MPK_OP_LINEAR, l, "down", m, 1, h);
      op.w = lw.wd; op.K = F;
      b.add(MPK_OP_ADD, l, "resid2", xo, 1, x1, m);
    }
    x = xo;
  }
  int lin = x;
  if (!(f & MPK_FUSE_NORM)) {
    int xnf = b.new_tensor(B, H);
    HostOp& op = b.add(MPK_OP_RMSNORM, -1, "final_norm", xnf, H, x);
    op.w2 = w ? w->final_norm : nullptr; op.f0 = c.rms_eps; op.K = H;
    lin = xnf;
  }
  int logits = b.new_tensor(B, V, /*external=*/true);
  {
    HostOp& op = b.add(MPK_OP_LINEAR, -1, "lm_head", logits, 1, lin);
    op.w = w ? w->lm_head : nullptr; op.K = H; op.flags |= TF_OUT_LOGITS;
    if (f & MPK_FUSE_NORM) { op.flags |= TF_PRO_NORM; op.w2 = w ? w->final_norm : nullptr; op.f0 = c.rms_eps; reads_x(op, false); }
  }
  if (o.greedy_loop) {
    // greedy sampling inside the graph: the tokens of the next step (one task per sequence);
    // with it the kernel can go round again without the host (multi-token launch)
    // T tasks per sequence: task (b, j) scans logits [V j / T, V (j+1) / T) of row b and leaves
    // (largest value, its index) in element (b, 2j .. 2j+1) of the output; the task of a row that
    // arrives last (counter p2 + b) picks the token from the T pairs
    const uint32_t T = o.tiles_sampling ? std::min(o.tiles_sampling, V) : std::max(1u, std::min(32u, V / 8192u));
    int ntok = b.new_tensor(B, 2 * T);
    HostOp& op = b.add(MPK_OP_ARGMAX, -1, "argmax", ntok, 2, logits);
    op.K = V;
    op.p1 = T;
  }
  return MPK_OK;
}

// ------------------------------------------------------------------ K2: decomposition
static void tile_bounds(const HostOp& op, uint32_t tile, uint32_t* b0, uint32_t* b1, uint32_t* c0,
                        uint32_t* c1) {
  uint32_t ib = tile / op.tc, ic = tile % op.tc, nu = op.cols / op.unit;
  *b0 = tile_begin(op.rows, op.tb, ib);
  *b1 = tile_begin(op.rows, op.tb, ib + 1);
  (void)nu;
  *c0 = col_tile_begin(op, ic) * op.unit;
  *c1 = col_tile_begin(op, ic + 1) * op.unit;
}

static void choose_partitions(const mpk_model_config& c, const mpk_compile_options& o,
                              HostGraph& g) {
  const uint32_t W = o.n_workers;
  for (auto& op : g.ops) {
    uint32_t nu = op.cols / op.unit;
    switch (op.kind) {
      case MPK_OP_LINEAR:
      case MPK_OP_GATEUP: {
        // One pass over the weights serves every batch row, so the batch is not split; rows are
        // split over the workers (the partition that minimises device-memory loading,
        // Section 4.1): each weight byte is read by exactly one task.
        uint32_t want = (op.flags & TF_OUT_LOGITS) ? (o.tiles_lm_head ? o.tiles_lm_head : W)
                                                   : (o.tiles_linear ? o.tiles_linear : W);
        uint32_t cap = std::max(1u, nu / 8);   // at least 8 output rows per task
        op.tb = 1;
        op.tc = std::max(1u, std::min(want, cap));
        if (op.flags & TF_SPLITK) { op.tc = W; break; }   // (row block, part) pairs, sized in build_ops
        // the matrix-core body (batch > 4) holds at most 512 weight rows per task: whole extra
        // rounds of tasks until the tiles fit (only when the tile count was not given)
        const bool given = (op.flags & TF_OUT_LOGITS) ? o.tiles_lm_head != 0 : o.tiles_linear != 0;
        const uint32_t per_row = (op.flags & TF_GATEUP) ? 2u : 1u;
        while (c.batch > 4 && !given && op.tc < cap && (nu + op.tc - 1) / op.tc * per_row > 512) op.tc = std::min(cap, op.tc + W);
        if (op.align_unit && nu % op.align_unit == 0) {
          // QKV projection: tiles that never straddle a head keep every tile in exactly one
          // attention group's producer set (no fork, hence no dummy tasks).  Every head gets the
          // same number of tiles, as many as `want` allows (at least 8 rows each); a head need
          // not divide evenly (tiles of 25 and 26 rows on the 8B shape: 240 tasks, where tiles
          // that divide head_dim gave 192).
          const uint32_t heads = nu / op.align_unit;
          op.seg_tiles = std::max(1u, std::min(want / heads, op.align_unit / 8));
          // A projection small enough to be pre-loaded whole (256 KB of weights per worker are
          // requested before the event) is bound by latency, not bandwidth: then it pays to leave
          // workers without a QKV task for the attention tasks that follow in the round-robin
          // order -- they request their cache rows while the projection still runs (measured on
          // the 8B shape: 192 + 64 tasks 3.47 ms, 240 + 64 tasks 3.62 ms per step).
          const uint64_t bytes_per_worker = (uint64_t)nu * op.K * 2u / std::max(1u, W);
          const uint32_t attn_tasks = c.batch * c.n_kv_heads * std::max(1u, o.attn_chunks);
          if (bytes_per_worker <= 256u * 1024u && attn_tasks < want && (want - attn_tasks) / heads >= 1)
            op.seg_tiles = std::min(op.seg_tiles, (want - attn_tasks) / heads);
          op.tc = heads * op.seg_tiles;
        }
        break;
      }
      case MPK_OP_ROPE:
      case MPK_OP_ATTN_PARTIAL:
        op.tb = op.rows;
        op.tc = nu;
        break;
      case MPK_OP_ATTN_MERGE:
        op.tb = op.rows;
        op.tc = c.n_kv_heads;
        break;
      case MPK_OP_ADD:
      case MPK_OP_SWIGLU:
        op.tb = op.rows;
        op.tc = std::max(1u, std::min(o.tiles_pointwise ? o.tiles_pointwise : 1u, nu));
        break;
      case MPK_OP_ARGMAX:
        op.tb = op.rows;
        op.tc = nu;
        break;
      case MPK_OP_ROUTER:   // one task: the per-expert token lists need every token's choice
      case MPK_OP_SERVE:    // one task: admission and the page stack are sequential decisions
        op.tb = 1;
        op.tc = 1;
        break;
      case MPK_OP_EXPERT:   // one element per expert task
        op.tb = 1;
        op.tc = nu;
        break;
      case MPK_OP_COMBINE:
        op.tb = op.rows;
        op.tc = std::max(1u, std::min(o.tiles_pointwise ? o.tiles_pointwise
                                                        : std::max(1u, W / op.rows), std::max(1u, nu / 256)));
        break;
      default:   // embed, rmsnorm: one task per batch row (needs the whole row)
        op.tb = op.rows;
        op.tc = 1;
    }
  }
  uint32_t base = 0;
  for (auto& op : g.ops) {
    op.task_base = base;
    base += op.tb * op.tc;
  }
}

// ------------------------------------------------------------------ K3: dependency analysis
// Regions of the input tensors that one task reads, from the operator's definition.
static void input_rects(const mpk_model_config& c, const HostOp& op, uint32_t tile,
                        std::vector<Rect>& out) {
  uint32_t b0, b1, c0, c1;
  tile_bounds(op, tile, &b0, &b1, &c0, &c1);
  const uint32_t d = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads, grp = nq / nkv;
  out.clear();
  switch (op.kind) {
    case MPK_OP_SERVE:   // request queue and metadata are not graph tensors
      break;
    case MPK_OP_EMBED:   // (serving graphs: the slot's token comes from the serving task)
      if (op.in_tensor >= 0) out.push_back({op.in_tensor, b0, b1, 0, 1});
      break;
    case MPK_OP_RMSNORM:
      out.push_back({op.in_tensor, b0, b1, 0, op.K});
      break;
    case MPK_OP_LINEAR:
    case MPK_OP_GATEUP:
      if (op.flags & TF_SPLITK) {
        // output columns [part x H + rows): the task reads its part of the input rows, and (if it
        // turns out to be the one that adds the parts up) the residual at its rows
        const uint32_t Hh = op.p1, part = c0 / Hh, klen = op.K / op.p0;
        out.push_back({op.in_tensor, b0, b1, part * klen, (part + 1) * klen});
        out.push_back({op.in2_tensor, b0, b1, c0 - part * Hh, c1 - part * Hh});
        break;
      }
      out.push_back({op.in_tensor, b0, b1, 0, UINT32_MAX});   // whole input rows
      if (op.flags & TF_EPI_RESID) {
        if (op.in2_kparts) {   // the residual is the sum of a split-K operator's parts
          const uint32_t Hh = op.cols;
          for (uint32_t part = 0; part < op.in2_kparts; ++part) out.push_back({op.in2_tensor, b0, b1, part * Hh + c0, part * Hh + c1});
        } else {
          out.push_back({op.in2_tensor, b0, b1, c0, c1});
        }
      }
      break;
    case MPK_OP_ROPE:
      out.push_back({op.in_tensor, b0, b1, c0, c1});   // whole heads: partners included
      break;
    case MPK_OP_ATTN_PARTIAL: {
      uint32_t per = grp * (d + 2), C = op.p1;
      // chunk tasks dealt to the sequences at run time: which sequence's query a task reads is
      // not known statically, so it depends on all of them
      if (op.flags & TF_ATTN_BALANCE) { b0 = 0; b1 = op.rows; }
      for (uint32_t u = c0 / per; u < c1 / per; ++u) {
        uint32_t gidx = u / C, ch = u % C;
        (void)ch;
        // every chunk task waits for the group's query heads AND this step's key/value of its KV
        // head: which chunk holds the appended row is a run-time fact, so the static set is the
        // superset (it also keeps all chunk tasks of a group on one event)
        out.push_back({op.in_tensor, b0, b1, gidx * grp * d, (gidx + 1) * grp * d});
        out.push_back({op.in_tensor, b0, b1, (nq + gidx) * d, (nq + gidx + 1) * d});
        out.push_back({op.in_tensor, b0, b1, (nq + nkv + gidx) * d, (nq + nkv + gidx + 1) * d});
      }
      break;
    }
    case MPK_OP_ATTN_MERGE: {
      uint32_t C = op.p1;
      for (uint32_t h = c0 / d; h < c1 / d; ++h) {
        uint32_t gidx = h / grp, j = h % grp;
        for (uint32_t ch = 0; ch < C; ++ch) {
          uint32_t base = ((gidx * C + ch) * grp + j) * (d + 2);
          out.push_back({op.in_tensor, b0, b1, base, base + d + 2});
        }
      }
      break;
    }
    case MPK_OP_ADD:
      out.push_back({op.in_tensor, b0, b1, c0, c1});
      out.push_back({op.in2_tensor, b0, b1, c0, c1});
      break;
    case MPK_OP_SWIGLU:
      out.push_back({op.in_tensor, b0, b1, c0, c1});
      out.push_back({op.in_tensor, b0, b1, op.p0 + c0, op.p0 + c1});
      break;
    case MPK_OP_ROUTER:   // every token's router output
      out.push_back({op.in_tensor, 0, UINT32_MAX, 0, UINT32_MAX});
      break;
    case MPK_OP_ARGMAX: {   // its share of the logits of its sequences
      const uint32_t T = op.p1, j0 = c0 / 2, j1 = c1 / 2;
      out.push_back({op.in_tensor, b0, b1, tile_begin(op.K, T, j0), tile_begin(op.K, T, j1)});
      break;
    }
    case MPK_OP_EXPERT:   // the meta-tensor + whatever routing sends here: statically everything
      out.push_back({op.in_tensor, 0, UINT32_MAX, 0, UINT32_MAX});
      out.push_back({op.in2_tensor, 0, UINT32_MAX, 0, UINT32_MAX});
      break;
    case MPK_OP_COMBINE:
      out.push_back({op.in_tensor, b0, b1, c0, c1});
      out.push_back({op.in2_tensor, 0, UINT32_MAX, 0, UINT32_MAX});
      out.push_back({op.in3_tensor, 0, UINT32_MAX, 0, UINT32_MAX});
      break;
  }
}

static void dependency_analysis(const mpk_model_config& c, HostGraph& g, PassInput& pi) {
  std::vector<int> producer_op(g.tensors.size(), -1);
  for (size_t i = 0; i < g.ops.size(); ++i) producer_op[g.ops[i].out_tensor] = (int)i;
  uint32_t n = 0;
  for (auto& op : g.ops) n += op.tb * op.tc;
  pi.n_real = n;
  pi.prod.assign(n, {});
  pi.op_of.resize(n);
  pi.tile_of_task.resize(n);
  std::vector<Rect> rects;
  for (size_t oi = 0; oi < g.ops.size(); ++oi) {
    const HostOp& op = g.ops[oi];
    for (uint32_t tile = 0; tile < op.tb * op.tc; ++tile) {
      uint32_t t = op.task_base + tile;
      pi.op_of[t] = (uint32_t)oi;
      pi.tile_of_task[t] = tile;
      input_rects(c, op, tile, rects);
      auto& P = pi.prod[t];
      for (const Rect& r : rects) {
        int po = producer_op[r.tensor];
        if (po < 0) continue;
        const HostOp& p = g.ops[po];
        uint32_t c1 = std::min(r.c1, p.cols), rb1 = std::min(r.b1, p.rows);
        if (r.b0 >= rb1 || r.c0 >= c1) continue;
        uint32_t nu = p.cols / p.unit;
        uint32_t ib0 = tile_of(p.rows, p.tb, r.b0), ib1 = tile_of(p.rows, p.tb, rb1 - 1);
        (void)nu;
        uint32_t ic0 = col_tile_of(p, r.c0 / p.unit), ic1 = col_tile_of(p, (c1 - 1) / p.unit);
        for (uint32_t ib = ib0; ib <= ib1; ++ib)
          for (uint32_t ic = ic0; ic <= ic1; ++ic) P.push_back(p.task_base + ib * p.tc + ic);
      }
      sort_unique(P);
    }
  }
}

// ------------------------------------------------------------------ K7 labels (operator level)
// Attention and expert tasks have a data-dependent duration -> JIT.  A downstream operator stays JIT unless each of
// its tasks waits for ALL tasks of every JIT operator it reads from (a global barrier with
// respect to the accumulated imbalance, Section 5.2).
static void label_ops(HostGraph& g, const PassInput& pi, std::vector<uint32_t>& op_jit) {
  op_jit.assign(g.ops.size(), 0);
  for (size_t oi = 0; oi < g.ops.size(); ++oi) {
    const HostOp& op = g.ops[oi];
    if (op.kind == MPK_OP_ATTN_PARTIAL || op.kind == MPK_OP_EXPERT) { op_jit[oi] = 1; continue; }
    bool jit = false;
    for (uint32_t tile = 0; tile < op.tb * op.tc && !jit; ++tile) {
      const auto& P = pi.prod[op.task_base + tile];
      std::map<uint32_t, uint32_t> per_op;
      for (uint32_t p : P) per_op[pi.op_of[p]]++;
      for (auto& kv : per_op)
        if (op_jit[kv.first] && kv.second != g.ops[kv.first].tb * g.ops[kv.first].tc) jit = true;
    }
    op_jit[oi] = jit ? 1u : 0u;
  }
  for (size_t oi = 0; oi < g.ops.size(); ++oi) g.ops[oi].jit = op_jit[oi];
}

// ------------------------------------------------------------------ task descriptors
static const float* act_ref(const HostGraph& g, int tensor) {
  if (tensor < 0) return nullptr;
  size_t off = g.tensors[tensor].offset;
  if (off == SIZE_MAX) return nullptr;
  return (const float*)(uintptr_t)((off + 1) * sizeof(float));   // relocated by the runtime
}

static void build_descs(const mpk_model_config& c, const mpk_kv_ptrs* kv, HostGraph& g) {
  g.descs.assign(g.tasks.size(), TaskDesc{});
  // elements of one layer's K (or V) cache: [batch][n_kv][max_seq][d], or the pool [pages][n_kv][page][d]
  const size_t kv_layer = g.opt.kv_page_size
                              ? (size_t)g.opt.kv_pages * c.n_kv_heads * g.opt.kv_page_size * c.head_dim
                              : (size_t)(g.opt.kv_batch ? g.opt.kv_batch : c.batch) * c.n_kv_heads * c.max_seq * c.head_dim;
  std::map<int, int32_t> route_event;   // layer -> the event its routing task triggers
  for (const HostTask& rt : g.tasks)
    if (rt.op != MPK_TASK_DUMMY_OP && g.ops[rt.op].kind == MPK_OP_ROUTER && rt.trig_event >= 0) route_event[g.ops[rt.op].layer] = rt.trig_event;
  for (size_t i = 0; i < g.tasks.size(); ++i) {
    const HostTask& ht = g.tasks[i];
    TaskDesc& t = g.descs[i];
    t.dep_event = ht.dep_event;
    t.trig_event = ht.trig_event;
    t.pad = i;   // own index in the linearized task list (trace slots are indexed by it)
    if (ht.op == MPK_TASK_DUMMY_OP) { t.kind = TK_DUMMY; continue; }
    const HostOp& op = g.ops[ht.op];
    tile_bounds(op, ht.tile, &t.b0, &t.b1, &t.c0, &t.c1);
    t.flags = op.flags | (ht.jit ? TF_JIT : 0);
    t.K = op.K;
    t.w = op.w; t.w2 = op.w2; t.f0 = op.f0; t.f1 = op.f1;
    t.p0 = op.p0; t.p1 = op.p1; t.p2 = op.p2; t.p3 = op.p3;
    t.in = act_ref(g, op.body_in_tensor >= 0 ? op.body_in_tensor : op.in_tensor);
    t.in2 = act_ref(g, op.side_out_tensor >= 0 ? op.side_out_tensor
                                               : (op.body_in2_tensor >= 0 ? op.body_in2_tensor : op.in2_tensor));
    t.out = const_cast<float*>(act_ref(g, op.out_tensor));
    {
      int it = op.body_in_tensor >= 0 ? op.body_in_tensor : op.in_tensor;
      t.ld_in = it >= 0 ? g.tensors[it].cols : 0;
    }
    t.ld_out = op.cols;
    switch (op.kind) {
      case MPK_OP_EMBED: t.kind = TK_EMBED; break;
      case MPK_OP_RMSNORM: t.kind = TK_RMSNORM; break;
      case MPK_OP_LINEAR:
      case MPK_OP_GATEUP: t.kind = TK_LINEAR; break;
      case MPK_OP_ROPE: t.kind = TK_ROPE; break;
      case MPK_OP_ATTN_PARTIAL: t.kind = TK_ATTN_PARTIAL; break;
      case MPK_OP_ATTN_MERGE: t.kind = TK_ATTN_MERGE; break;
      case MPK_OP_ADD: t.kind = TK_ADD; break;
      case MPK_OP_SWIGLU: t.kind = TK_SWIGLU; break;
      case MPK_OP_ROUTER: t.kind = TK_MOE_ROUTE; break;
      case MPK_OP_EXPERT: t.kind = TK_MOE_EXPERT; break;
      case MPK_OP_COMBINE: t.kind = TK_MOE_COMBINE; break;
      case MPK_OP_ARGMAX: t.kind = TK_ARGMAX; break;
      case MPK_OP_SERVE: t.kind = TK_SERVE; break;
    }
    if (op.flags & TF_SPLITK) {
      const uint32_t Hh = op.p1, parts = op.p0, part = t.c0 / Hh, klen = op.K / parts;
      t.K = klen;
      t.p1 = op.K;                                   // weight row length
      t.p3 = parts | (part << 8);
      t.p2 = g.n_group_counters_attn + op.p2 + (t.c0 - part * Hh) / (t.c1 - t.c0);   // row block's arrival counter
      t.w = op.w ? (const void*)((const uint16_t*)op.w + (size_t)part * klen) : nullptr;
      t.in = (const float*)((const char*)act_ref(g, op.in_tensor) + (size_t)part * klen * sizeof(float));
      t.in2 = act_ref(g, op.in2_tensor);             // residual [B][H]
      t.aux0 = (void*)act_ref(g, op.side_out_tensor);   // the real output [B][H]; relocated by the runtime
    }
    if (op.kind == MPK_OP_ARGMAX) t.p2 = g.n_group_counters_attn + g.n_splitk_counters;   // first sampling counter (+ sequence)
    if (op.kind == MPK_OP_ROUTER || op.kind == MPK_OP_EXPERT || op.kind == MPK_OP_COMBINE) {
      t.in = act_ref(g, op.data_in);
      t.in2 = act_ref(g, op.data_in2);
      t.out = const_cast<float*>(act_ref(g, op.data_out));
      t.aux0 = (void*)act_ref(g, op.data_aux);   // relocated by the runtime like in / in2 / out
      t.ld_in = g.tensors[op.data_in].cols;
      t.ld_out = g.tensors[op.data_out].cols;
      // second-stage expert task: the event the layer's routing task triggers (+ 1), behind which
      // the meta-tensor may be read -- the task requests its first weights before its own event
      if (op.kind == MPK_OP_EXPERT && !(op.flags & TF_GATEUP)) {
        auto it = route_event.find(op.layer);
        if (it != route_event.end()) t.aux1 = (void*)(uintptr_t)(it->second + 1);
      }
    }
    if (op.kind == MPK_OP_ROPE || op.kind == MPK_OP_ATTN_PARTIAL) {
      if (kv && kv->k && kv->v) {
        t.aux0 = (uint16_t*)kv->k + (size_t)op.p0 * kv_layer;
        t.aux1 = (uint16_t*)kv->v + (size_t)op.p0 * kv_layer;
      }
    }
  }
}

static uint32_t lds_requirement(const mpk_model_config& c, HostGraph& g, uint32_t C) {
  size_t need = 0;
  const uint32_t grp = c.n_q_heads / c.n_kv_heads;
  const uint32_t nb = c.batch <= 2 ? c.batch : (c.batch <= 4 ? 4u : 8u);   // body template sizes
  // linear tasks: staged input rows | per-row results | residual slice | partial sums of squares
  uint32_t rows_max = 0;
  for (auto& op : g.ops) {
    if (op.kind != MPK_OP_LINEAR && op.kind != MPK_OP_GATEUP) continue;
    uint32_t nu = op.cols / op.unit, per = col_tile_max_units(op) * op.unit;
    rows_max = std::max(rows_max, per * ((op.flags & TF_GATEUP) ? 2u : 1u));
  }
  g.lin_rows_max = rows_max;
  uint32_t res_rows = 0;   // columns of the largest task that adds a residual
  for (auto& op : g.ops) {
    if ((op.kind != MPK_OP_LINEAR && op.kind != MPK_OP_GATEUP) || !(op.flags & TF_EPI_RESID)) continue;
    uint32_t nu = op.cols / op.unit;
    res_rows = std::max(res_rows, col_tile_max_units(op) * op.unit);
  }
  g.lin_res_rows_max = res_rows;
  for (auto& op : g.ops) {
    size_t f = 0;
    if (op.kind == MPK_OP_LINEAR || op.kind == MPK_OP_GATEUP) {
      if (c.batch <= 4) {
        f = (size_t)nb * ((op.K + 4095u) / 4096u * 4096u) + 2 * (size_t)rows_max * nb + 8 * nb;
      } else {
        // matrix-core body: the staged fp32 input, one chunk (reused for the per-wavefront
        // partial tiles) | residual slice | sums of squares | 1/rms per row
        f = (size_t)mfma_x_floats(c.batch) + (size_t)res_rows * 16 + 10 * 16;   // ... | split-K arrival flag
      }
    }
    else if (op.kind == MPK_OP_EXPERT) {
      f = (size_t)moe_x_floats(c.batch) + 8 * 16 + 32   // input tiles | sums of squares | staged row lists
          + 2 + 3 * (size_t)c.n_experts + (size_t)c.batch * c.top_k;   // | the task's copy of the meta-tensor
    }
    else if (op.kind == MPK_OP_ROUTER)
      f = (size_t)c.batch * c.top_k * 2 + (size_t)c.n_experts * (3 + 16) + 64;   // pairs | per-expert counts, offsets, masks, pair table
    else if (op.kind == MPK_OP_ATTN_PARTIAL)
      f = (size_t)grp * c.head_dim                                        // q
          + (size_t)(kThreads * 8 / c.head_dim) * grp * (c.head_dim + 4) + 16 + 64;   // partials per position slot (register-resident body; the other keeps one per wavefront)
    if (op.kind == MPK_OP_ATTN_PARTIAL && g.opt.kv_page_size)   // paged cache: + the chunk's page numbers
      f += c.max_seq / g.opt.kv_page_size;
    need = std::max(need, f);
  }
  size_t bytes = (need + kLdsReduceFloats + kLdsCtrlFloats) * sizeof(float);   // + the control words
  return (uint32_t)std::max<size_t>(bytes, kMinLdsBytes);
}

static mpk_status validate(const mpk_model_config& c, const mpk_weight_ptrs* w,
                           const mpk_kv_ptrs* kv, const mpk_compile_options& o) {
  if (c.struct_size != sizeof(mpk_model_config)) { set_error("mpk_model_config.struct_size is %u, expected %zu", c.struct_size, sizeof(mpk_model_config)); return MPK_ERR_INVALID_ARG; }
  if (!c.n_layers || !c.hidden || !c.n_q_heads || !c.n_kv_heads || !c.head_dim || !c.vocab || !c.batch || !c.max_seq) { set_error("a model dimension is zero"); return MPK_ERR_INVALID_ARG; }
  if (c.flags & ~MPK_MODEL_QK_NORM) { set_error("unknown mpk_model_config.flags bits"); return MPK_ERR_INVALID_ARG; }
  const bool moe = c.n_experts != 0;
  if (moe) {
    if (!c.top_k || !c.expert_ffn || c.top_k > c.n_experts) { set_error("mixture-of-experts: top_k and expert_ffn must be non-zero and top_k <= n_experts"); return MPK_ERR_INVALID_ARG; }
    if (c.n_experts > kMoeMaxExperts || c.top_k > kMoeMaxTopK || c.batch * c.top_k > kMoeMaxPairs) { set_error("mixture-of-experts: at most %u experts, top_k %u, batch x top_k %u", kMoeMaxExperts, kMoeMaxTopK, kMoeMaxPairs); return MPK_ERR_UNSUPPORTED; }
    if (o.tiles_moe > 4096) { set_error("tiles_moe %u too large (max 4096)", o.tiles_moe); return MPK_ERR_INVALID_ARG; }
    if (c.expert_ffn % 8 || c.expert_ffn < 32 || c.hidden % 16) { set_error("mixture-of-experts: expert_ffn must be a multiple of 8 (at least 32) and hidden a multiple of 16"); return MPK_ERR_UNSUPPORTED; }
  } else {
    if (c.top_k || c.expert_ffn) { set_error("top_k / expert_ffn set without n_experts"); return MPK_ERR_INVALID_ARG; }
    if (!c.ffn) { set_error("ffn is zero"); return MPK_ERR_INVALID_ARG; }
  }
  if (c.batch > 4) {
    // the matrix-core body addresses a weight matrix with 32-bit byte offsets from its first row
    const uint64_t rows = std::max<uint64_t>({c.vocab, 2ull * c.ffn, (uint64_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, c.hidden});
    const uint64_t inner = std::max<uint64_t>({c.hidden, c.ffn, (uint64_t)c.n_q_heads * c.head_dim});
    if (rows * inner * 2ull >= (1ull << 32)) { set_error("a weight matrix of 4 GB or more is unsupported at batch sizes above 4"); return MPK_ERR_UNSUPPORTED; }
  }
  if (c.head_dim != 64 && c.head_dim != 128) { set_error("head_dim %u unsupported (64 or 128)", c.head_dim); return MPK_ERR_UNSUPPORTED; }
  if (c.n_q_heads % c.n_kv_heads) { set_error("n_q_heads must be a multiple of n_kv_heads"); return MPK_ERR_UNSUPPORTED; }
  {
    uint32_t grp = c.n_q_heads / c.n_kv_heads;
    if (grp != 1 && grp != 2 && grp != 4 && grp != 8) { set_error("%u query heads per KV head unsupported (1, 2, 4 or 8)", grp); return MPK_ERR_UNSUPPORTED; }
  }
  if (c.hidden % 8 || (!moe && c.ffn % 8) || (c.n_q_heads * c.head_dim) % 8) { set_error("hidden, ffn and n_q*head_dim must be multiples of 8"); return MPK_ERR_UNSUPPORTED; }
  if (c.batch > 16) { set_error("batch %u unsupported by the dense linear bodies (max 16)", c.batch); return MPK_ERR_UNSUPPORTED; }
  if (o.greedy_loop > 2) { set_error("greedy_loop must be 0, 1 or 2"); return MPK_ERR_INVALID_ARG; }
  if (o.debug_flags & ~(MPK_DEBUG_TRACE | MPK_DEBUG_POISON | MPK_DEBUG_JITTER | MPK_DEBUG_LOSE_NOTIFY)) { set_error("unknown debug_flags bits"); return MPK_ERR_INVALID_ARG; }
  if (o.kv_batch != 0 && o.kv_batch < c.batch) { set_error("kv_batch %u is below batch %u", o.kv_batch, c.batch); return MPK_ERR_INVALID_ARG; }
  if (o.kv_page_size) {
    const uint32_t ps = o.kv_page_size;
    if (ps < 8 || (ps & (ps - 1)) || c.max_seq % ps) { set_error("kv_page_size %u must be a power of two >= 8 that divides max_seq %u", ps, c.max_seq); return MPK_ERR_INVALID_ARG; }
    if (!(o.fusion & MPK_FUSE_ROPE)) { set_error("a paged KV cache needs MPK_FUSE_ROPE (the attention tasks append the new rows)"); return MPK_ERR_UNSUPPORTED; }
    if (o.kv_batch) { set_error("kv_batch does not apply to a paged KV cache"); return MPK_ERR_INVALID_ARG; }
    if (o.kv_pages < c.batch + 1u) { set_error("kv_pages %u: a paged cache needs more pages than batch slots (%u)", o.kv_pages, c.batch); return MPK_ERR_INVALID_ARG; }
    if ((uint64_t)o.kv_pages * c.n_kv_heads * ps * c.head_dim >= (1ull << 40)) { set_error("kv_pages %u: pool too large", o.kv_pages); return MPK_ERR_UNSUPPORTED; }
  } else if (o.kv_pages) { set_error("kv_pages without kv_page_size"); return MPK_ERR_INVALID_ARG; }
  if (o.serving > 1) { set_error("serving must be 0 or 1"); return MPK_ERR_INVALID_ARG; }
  if (o.serving) {
    if (!o.greedy_loop || !o.kv_page_size) { set_error("serving needs greedy_loop = 1 and a paged KV cache (kv_page_size)"); return MPK_ERR_INVALID_ARG; }
    if (o.n_sched_wgs && !o.force_aot) { set_error("serving is only supported without scheduler workgroups"); return MPK_ERR_UNSUPPORTED; }
  }
  if (o.fusion & ~(MPK_FUSE_NORM | MPK_FUSE_RESID | MPK_FUSE_SWIGLU | MPK_FUSE_MERGE | MPK_FUSE_ROPE)) { set_error("unknown fusion bits"); return MPK_ERR_INVALID_ARG; }
  if (!o.host_only) {
    if (!w || !kv || !w->layers) { set_error("weights / kv pointers are NULL"); return MPK_ERR_INVALID_ARG; }
    auto bad = [](const void* p) { return p == nullptr || ((uintptr_t)p & 15u); };
    if (bad(w->embed) || bad(w->final_norm) || bad(w->lm_head) || bad(kv->k) || bad(kv->v)) { set_error("a model-level pointer is NULL or not 16-byte aligned"); return MPK_ERR_INVALID_ARG; }
    for (uint32_t l = 0; l < c.n_layers; ++l) {
      const mpk_layer_weights& lw = w->layers[l];
      if ((c.flags & MPK_MODEL_QK_NORM) && (bad(lw.q_norm) || bad(lw.k_norm))) { set_error("layer %u: q_norm / k_norm pointer is NULL or not 16-byte aligned", l); return MPK_ERR_INVALID_ARG; }
      if (bad(lw.attn_norm) || bad(lw.wqkv) || bad(lw.wo) || bad(lw.mlp_norm) ||
          (moe ? (bad(lw.router) || bad(lw.expert_wgu) || bad(lw.expert_wd)) : (bad(lw.wgu) || bad(lw.wd)))) { set_error("layer %u: a weight pointer is NULL or not 16-byte aligned", l); return MPK_ERR_INVALID_ARG; }
    }
  }
  return MPK_OK;
}

// Tiles sized by the speed of the worker that runs them (option worker_weight_permille: the eight
// XCDs of the GPU do not stream equally fast, and an operator ends with its slowest task).  Which
// worker runs which tile is only known after linearization and pre-enqueue, but it does not depend
// on the tile SIZES: the graph is built once with even tiles, the assignment is read off, and the
// graph is built again with the weighted column tiles.  Eligible: linear operators of the vector
// body (batch <= 4) with one row of tiles, no head alignment and no input split, every task
// ahead-of-time.
using TileWorkers = std::vector<std::vector<int32_t>>;   // [operator][tile] -> worker, empty = not eligible
static void apply_worker_weights(const mpk_compile_options& o, const TileWorkers& tw, HostGraph& g) {
  for (size_t oi = 0; oi < g.ops.size() && oi < tw.size(); ++oi) {
    HostOp& op = g.ops[oi];
    if (tw[oi].empty() || tw[oi].size() != op.tc) continue;
    const uint32_t nu = op.cols / op.unit;
    std::vector<double> wsum(op.tc + 1, 0.0);
    for (uint32_t i = 0; i < op.tc; ++i) wsum[i + 1] = wsum[i] + (double)std::max(1u, o.worker_weight_permille[(uint32_t)tw[oi][i] & 7u]);
    op.col_begin.assign(op.tc + 1, 0);
    for (uint32_t i = 1; i < op.tc; ++i) {
      uint32_t b = (uint32_t)std::llround((double)nu * wsum[i] / wsum[op.tc]);
      b = std::max(b, op.col_begin[i - 1] + 1u);       // never an empty tile
      b = std::min(b, nu - (op.tc - i));
      op.col_begin[i] = b;
    }
    op.col_begin[op.tc] = nu;
  }
}

// LDS floats a batch-1 linear task of this operator needs below the page area.
static size_t lin_task_floats_b1(const HostGraph& g, const HostOp& op) {
  return (size_t)((op.K + 4095u) / 4096u * 4096u) + 2 * (size_t)g.lin_rows_max + 8;
}
static bool page_capable(const mpk_model_config& c, const mpk_compile_options& o) {
  return c.batch == 1 && !o.no_lds_pages && !o.no_preload && o.n_sched_wgs == 0 && o.launch_mode == MPK_LAUNCH_MEGA && true;
}

// Which tasks get their first half blocks pre-loaded into the LDS pages by the task before them in
// their worker's list (Section 5.3, pre-loading across tasks).  A pair (T, N) of consecutive linear
// tasks of one worker qualifies when T comes right after another linear task (so the worker is not
// one that just ran an attention task: it has the whole attention phase to wait through), T and N
// both leave room for the pages in LDS, and N is long enough to gain (more than two half blocks
// per wavefront).  Returns, per task of the linearized list, 0, TF_PAGE_NEXT or TF_PAGE_READY.
static std::vector<uint16_t> page_plan(const mpk_model_config& c, const mpk_compile_options& o, const HostGraph& g) {
  std::vector<uint16_t> plan(g.tasks.size(), 0);
  if (!page_capable(c, o)) return plan;
  const size_t room = (160 * 1024) / sizeof(float) - kLdsReduceFloats - kLdsCtrlFloats - kLinPagesFloats;
  auto lin_op = [&](uint32_t ti) -> const HostOp* {
    const HostTask& t = g.tasks[ti];
    if (t.op == MPK_TASK_DUMMY_OP || t.jit) return nullptr;
    const HostOp& op = g.ops[t.op];
    return (op.kind == MPK_OP_LINEAR || op.kind == MPK_OP_GATEUP) ? &op : nullptr;
  };
  for (uint32_t w = 0; w + 1 < g.aot_off.size(); ++w) {
    for (uint32_t qi = g.aot_off[w] + 1; qi + 1 < g.aot_off[w + 1]; ++qi) {
      const HostOp *prev = lin_op(g.aot[qi - 1]), *cur = lin_op(g.aot[qi]), *next = lin_op(g.aot[qi + 1]);
      if (!prev || !cur || !next) continue;
      if (prev->layer != cur->layer || cur->layer != next->layer || cur->layer < 0) continue;
      // T is short (fits its two register buffers: nothing of its own left to stream while it waits)
      const uint64_t cur_rows = (uint64_t)cur->cols * ((cur->flags & TF_GATEUP) ? 2u : 1u) / cur->tc;
      const uint64_t next_rows = (uint64_t)next->cols * ((next->flags & TF_GATEUP) ? 2u : 1u) / next->tc;
      if (cur_rows * cur->K * 2 > 256 * 1024) continue;
      if (next->K > 4096 || next_rows < 48 || (next->flags & TF_SPLITK) || next->seg_tiles) continue;
      if (lin_task_floats_b1(g, *cur) > room || lin_task_floats_b1(g, *next) > room) continue;
      plan[g.aot[qi]] |= TF_PAGE_NEXT;
      plan[g.aot[qi + 1]] |= TF_PAGE_READY;
    }
  }
  return plan;
}

// Column tiles of the operators whose tasks are partly pre-loaded into LDS pages: a task with its
// first kLinPageUnits weight rows already on the chip when its event fires gets that many more
// rows than a task without, so that both have the same amount left to stream.
static void apply_page_sizes(const std::vector<std::vector<uint8_t>>& ready, HostGraph& g) {
  for (size_t oi = 0; oi < g.ops.size() && oi < ready.size(); ++oi) {
    HostOp& op = g.ops[oi];
    if (ready[oi].empty() || ready[oi].size() != op.tc || !op.col_begin.empty()) continue;
    const uint32_t n_ready = (uint32_t)std::count(ready[oi].begin(), ready[oi].end(), (uint8_t)1);
    if (n_ready == 0 || n_ready == op.tc) continue;          // all alike: the even split is right
    const uint32_t nu = op.cols / op.unit;
    const uint32_t bonus = kLinPageUnits / ((op.flags & TF_GATEUP) ? 2u : 1u) / std::max(1u, op.unit);
    const uint64_t total = (uint64_t)nu + (uint64_t)bonus * (op.tc - n_ready);
    const uint32_t x = (uint32_t)(total / op.tc);            // size of a pre-loaded tile
    if (x <= bonus + 8) continue;
    uint32_t rem = (uint32_t)(total % op.tc);                 // left-over units: one more for the first tiles
    op.col_begin.assign(op.tc + 1, 0);
    for (uint32_t i = 0; i < op.tc; ++i) {
      uint32_t sz = ready[oi][i] ? x : x - bonus;
      if (rem) { ++sz; --rem; }
      op.col_begin[i + 1] = std::min(nu, op.col_begin[i] + sz);
    }
    op.col_begin[op.tc] = nu;
  }
}

struct SecondPass {
  const TileWorkers* tile_workers = nullptr;
  const std::vector<std::vector<uint8_t>>* page_ready = nullptr;   // [operator][tile]
};
static mpk_status build_model_graph_pass(const mpk_model_config& cfg, const mpk_weight_ptrs* w,
                                         const mpk_kv_ptrs* kv, const mpk_compile_options& opt_in,
                                         const SecondPass& sp, HostGraph& g);

mpk_status build_model_graph(const mpk_model_config& cfg, const mpk_weight_ptrs* w,
                             const mpk_kv_ptrs* kv, const mpk_compile_options& opt_in,
                             HostGraph& g) {
  mpk_status st = build_model_graph_pass(cfg, w, kv, opt_in, SecondPass{}, g);
  if (st != MPK_OK) return st;
  bool weighted = false;
  for (int k = 0; k < 8; ++k) weighted = weighted || (opt_in.worker_weight_permille[k] != 0 && opt_in.worker_weight_permille[k] != opt_in.worker_weight_permille[0]);
  weighted = weighted && cfg.batch <= 4;
  // tiles that will find their first rows in the LDS pages
  std::vector<std::vector<uint8_t>> ready(g.ops.size());
  bool paged = false;
  {
    const std::vector<uint16_t> plan = page_plan(cfg, g.opt, g);
    for (size_t i = 0; i < g.tasks.size(); ++i) {
      if (!(plan[i] & TF_PAGE_READY)) continue;
      const HostTask& t = g.tasks[i];
      if (ready[t.op].empty()) ready[t.op].assign(g.ops[t.op].tc, 0);
      ready[t.op][t.tile] = 1;
      paged = true;
    }
  }
  if (!weighted && !paged) return MPK_OK;
  TileWorkers tw(g.ops.size());
  for (size_t oi = 0; oi < g.ops.size(); ++oi) {
    const HostOp& op = g.ops[oi];
    if ((op.kind != MPK_OP_LINEAR && op.kind != MPK_OP_GATEUP) || op.seg_tiles || (op.flags & TF_SPLITK) || op.tb != 1 || op.tc < 2 || op.jit) continue;
    // A task deals its rows to eight wavefronts in pairs: a tile of 8 pairs that grows to 9 doubles
    // one wavefront's share (measured: the 16-row tiles of the 8B shape's O and down projections
    // got 3 us slower).  Only tiles of at least four pairs per wavefront are resized.
    if ((uint64_t)(op.cols / op.unit) * op.unit * ((op.flags & TF_GATEUP) ? 2u : 1u) / op.tc < 64u) continue;
    if (weighted && ready[oi].empty()) tw[oi].assign(op.tc, -1);
  }
  for (const HostTask& t : g.tasks)
    if (t.op != MPK_TASK_DUMMY_OP && !tw[t.op].empty()) tw[t.op][t.tile] = t.worker;
  for (auto& v : tw)
    if (std::find(v.begin(), v.end(), -1) != v.end()) v.clear();   // a task without a fixed worker: leave the operator alone
  HostGraph g2;
  SecondPass sp;
  sp.tile_workers = &tw;
  sp.page_ready = &ready;
  st = build_model_graph_pass(cfg, w, kv, opt_in, sp, g2);
  if (st != MPK_OK) return st;
  if (g2.tasks.size() != g.tasks.size()) { set_error("task list changed between the two compile passes"); return MPK_ERR_INTERNAL; }
  for (size_t i = 0; i < g.tasks.size(); ++i)   // the assignment the sizes were computed for must be the one that came out
    if (g.tasks[i].op != g2.tasks[i].op || g.tasks[i].tile != g2.tasks[i].tile || g.tasks[i].worker != g2.tasks[i].worker) {
      set_error("worker assignment changed between the two compile passes");
      return MPK_ERR_INTERNAL;
    }
  g = std::move(g2);
  return MPK_OK;
}

static mpk_status build_model_graph_pass(const mpk_model_config& cfg, const mpk_weight_ptrs* w,
                                         const mpk_kv_ptrs* kv, const mpk_compile_options& opt_in,
                                         const SecondPass& sp, HostGraph& g) {
  mpk_compile_options opt = opt_in;
  mpk_status st = validate(cfg, w, kv, opt);
  if (st != MPK_OK) return st;
  if (opt.n_workers == 0) { set_error("n_workers unresolved"); return MPK_ERR_INTERNAL; }
  uint32_t C = opt.attn_chunks;
  if (C == 0) {
    // About one attention task per worker, but no chunk shorter than 128 cache positions (each
    // task has a fixed cost: event wait, query staging, the merge of its partial result).
    // Measured: C2 (8 pairs, 1088 positions) is fastest with 8 chunks, C3 (64 pairs) with 4.
    const uint32_t pairs = cfg.batch * cfg.n_kv_heads;
    C = (opt.n_workers + pairs - 1) / pairs;
    C = std::min(C, std::max(1u, cfg.max_seq / 128u));
    C = std::max(1u, std::min(C, 64u));
  }
  if (C > 64) { set_error("attn_chunks %u too large (max 64)", C); return MPK_ERR_INVALID_ARG; }
  opt.attn_chunks = C;
  g.cfg = cfg;
  g.opt = opt;
  st = build_ops(cfg, w, opt, C, g);
  if (st != MPK_OK) return st;
  choose_partitions(cfg, opt, g);
  if (sp.page_ready) apply_page_sizes(*sp.page_ready, g);
  if (sp.tile_workers) apply_worker_weights(opt, *sp.tile_workers, g);
  g.n_group_counters_attn = cfg.n_layers * cfg.batch * cfg.n_kv_heads;
  g.n_group_counters = g.n_group_counters_attn + g.n_splitk_counters + (opt.greedy_loop ? cfg.batch : 0u);   // + one per sequence for the sampling tasks
  g.inv_freq.resize(cfg.head_dim / 2);
  for (uint32_t i = 0; i < cfg.head_dim / 2; ++i)
    g.inv_freq[i] = std::pow((double)cfg.rope_theta, -2.0 * (double)i / (double)cfg.head_dim);
  PassInput pi;
  dependency_analysis(cfg, g, pi);
  label_ops(g, pi, pi.op_jit);   // labels follow the paper's rule on the full dependency sets
  if (opt.transitive_reduction) g.stats.n_pairs_removed = transitive_reduction(pi, g.ops);
  // count pairs before reduction for the statistics
  st = run_passes(pi, opt, g);
  if (st != MPK_OK) return st;
  g.stats.n_pair_deps += g.stats.n_pairs_removed;
  build_descs(cfg, kv, g);
  g.lds_bytes = lds_requirement(cfg, g, C);
  if (sp.page_ready) {   // (second pass: the tile sizes already account for the pages)
    const std::vector<uint16_t> plan = page_plan(cfg, opt, g);
    bool any = false;
    for (size_t i = 0; i < g.tasks.size(); ++i) {
      g.descs[i].flags |= plan[i];
      any = any || plan[i];
      if ((plan[i] & TF_PAGE_READY) && !(*sp.page_ready)[g.tasks[i].op][g.tasks[i].tile]) { set_error("page plan changed between the two compile passes"); return MPK_ERR_INTERNAL; }
    }
    if (any) {   // the pages sit at the top of the 160 KB
      g.lin_page_off = (uint32_t)((160 * 1024) / sizeof(float) - kLdsReduceFloats - kLdsCtrlFloats - kLinPagesFloats);
      g.lds_bytes = 160 * 1024;
    }
  }
  if (cfg.batch > 4 && g.lin_rows_max > 512) { set_error("a linear task would own %u weight rows; the batch >= 5 body handles at most 512: raise tiles_linear / tiles_lm_head", g.lin_rows_max); return MPK_ERR_UNSUPPORTED; }
  if (g.lds_bytes > 160 * 1024 && !opt.host_only) { set_error("task bodies need %u bytes of LDS (> 160 KB): batch x input length too large", g.lds_bytes); return MPK_ERR_UNSUPPORTED; }
  // statistics
  g.stats.struct_size = sizeof(mpk_stats);
  g.stats.n_ops = (uint32_t)g.ops.size();
  g.stats.lds_bytes = g.lds_bytes;
  g.stats.act_bytes = g.arena_floats * sizeof(float);
  uint64_t wb = (uint64_t)cfg.batch * cfg.hidden * 2 + (uint64_t)cfg.hidden * 2 +
                (uint64_t)cfg.vocab * cfg.hidden * 2;
  uint64_t qkv_rows = (uint64_t)(cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim;
  wb += (uint64_t)cfg.n_layers * 2 * (2ull * cfg.hidden + qkv_rows * cfg.hidden +
                                      (uint64_t)cfg.hidden * cfg.n_q_heads * cfg.head_dim +
                                      (cfg.n_experts ? (uint64_t)cfg.n_experts * cfg.hidden
                                                     : 3ull * cfg.ffn * cfg.hidden));
  g.stats.weight_bytes = wb;
  g.stats.expert_bytes = cfg.n_experts ? 3ull * cfg.expert_ffn * cfg.hidden * 2 : 0;
  g.stats.kv_row_bytes = (uint64_t)cfg.n_layers * 2 * cfg.n_kv_heads * cfg.head_dim * 2;
  return MPK_OK;
}

mpk_status build_dag_graph(uint32_t n_tasks, const uint32_t* pairs, size_t n_pairs,
                           const mpk_compile_options& opt, HostGraph& g) {
  if (n_tasks == 0 || (!pairs && n_pairs)) { set_error("empty DAG"); return MPK_ERR_INVALID_ARG; }
  if (opt.n_workers == 0) { set_error("n_workers unresolved"); return MPK_ERR_INTERNAL; }
  PassInput pi;
  pi.n_real = n_tasks;
  pi.prod.assign(n_tasks, {});
  pi.op_of.assign(n_tasks, 0);
  pi.tile_of_task.resize(n_tasks);
  std::iota(pi.tile_of_task.begin(), pi.tile_of_task.end(), 0u);
  for (size_t i = 0; i < n_pairs; ++i) {
    uint32_t a = pairs[2 * i], b = pairs[2 * i + 1];
    if (a >= n_tasks || b >= n_tasks || a == b) { set_error("pair %zu (%u -> %u) out of range", i, a, b); return MPK_ERR_INVALID_ARG; }
    pi.prod[b].push_back(a);
  }
  for (auto& P : pi.prod) sort_unique(P);
  g.opt = opt;
  HostOp op{};
  op.kind = MPK_OP_ADD; op.layer = -1; op.name = "dag"; op.tb = 1; op.tc = n_tasks;
  op.rows = 1; op.cols = n_tasks; op.unit = 1; op.in_tensor = op.in2_tensor = op.out_tensor = -1;
  g.ops.push_back(op);
  mpk_status st = run_passes(pi, opt, g);
  if (st != MPK_OK) return st;
  g.stats.struct_size = sizeof(mpk_stats);
  g.stats.n_ops = 1;
  return MPK_OK;
}

// ------------------------------------------------------------------ export
size_t export_size(const HostGraph& g) {
  size_t n = sizeof(mpk_export_header) + g.ops.size() * sizeof(mpk_export_op) +
             g.tasks.size() * sizeof(mpk_export_task) + g.events.size() * sizeof(mpk_export_event) +
             (g.aot_off.size() + g.aot.size()) * sizeof(uint32_t) + sizeof(uint32_t);
  for (auto& op : g.ops)
    if (!op.col_begin.empty()) n += (2 + op.col_begin.size()) * sizeof(uint32_t);
  return n;
}

void export_graph(const HostGraph& g, void* buf) {
  char* p = (char*)buf;
  mpk_export_header h{};
  h.magic = MPK_EXPORT_MAGIC; h.version = 2;
  h.n_ops = (uint32_t)g.ops.size(); h.n_tasks = (uint32_t)g.tasks.size();
  h.n_events = (uint32_t)g.events.size(); h.n_workers = g.opt.n_workers;
  h.n_sched_wgs = g.opt.n_sched_wgs; h.start_event = g.start_event;
  h.terminal_event = g.terminal_event; h.n_real_tasks = g.n_real; h.fusion = g.opt.fusion;
  memcpy(p, &h, sizeof(h)); p += sizeof(h);
  for (auto& op : g.ops) {
    mpk_export_op e{op.kind, op.layer, op.tb, op.tc, op.tb * op.tc, op.jit, op.rows, op.cols};
    memcpy(p, &e, sizeof(e)); p += sizeof(e);
  }
  for (auto& t : g.tasks) {
    mpk_export_task e{t.op, t.tile, t.dep_event, t.trig_event, t.worker, t.jit};
    memcpy(p, &e, sizeof(e)); p += sizeof(e);
  }
  for (auto& ev : g.events) {
    mpk_export_event e{ev.required, ev.first, ev.last, ev.flags};
    memcpy(p, &e, sizeof(e)); p += sizeof(e);
  }
  memcpy(p, g.aot_off.data(), g.aot_off.size() * 4); p += g.aot_off.size() * 4;
  memcpy(p, g.aot.data(), g.aot.size() * 4); p += g.aot.size() * 4;
  // operators with explicit column tiles: count, then per operator its index, the number of
  // boundaries and the boundaries in columns
  uint32_t n_explicit = 0;
  for (auto& op : g.ops) n_explicit += op.col_begin.empty() ? 0u : 1u;
  memcpy(p, &n_explicit, 4); p += 4;
  for (size_t oi = 0; oi < g.ops.size(); ++oi) {
    const HostOp& op = g.ops[oi];
    if (op.col_begin.empty()) continue;
    const uint32_t hdr[2] = {(uint32_t)oi, (uint32_t)op.col_begin.size()};
    memcpy(p, hdr, 8); p += 8;
    for (uint32_t b : op.col_begin) { const uint32_t c = b * op.unit; memcpy(p, &c, 4); p += 4; }
  }
}

}  // namespace mpk

extern "C" mpk_status mpk_moe_task_share(uint32_t n_active, uint32_t tiles_per_expert, uint32_t n_tasks, uint32_t task,
                                         uint32_t* first, uint32_t* last) {
  if (!first || !last || n_tasks == 0 || task >= n_tasks || tiles_per_expert == 0) {
    mpk::set_error("mpk_moe_task_share: null pointer, no tasks, task out of range or no tiles");
    return MPK_ERR_INVALID_ARG;
  }
  mpk::moe_task_share(n_active, tiles_per_expert, n_tasks, task, first, last);
  return MPK_OK;
}
