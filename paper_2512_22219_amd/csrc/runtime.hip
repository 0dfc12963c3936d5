// Host side of the runtime: the C ABI entry points (compile, launch, status, export, graph sets).
// The kernels live in kernels.h and are instantiated by variants.hip, one specialised set per
// translation unit; this file only picks a set and launches it.
#include <algorithm>

#include "kernels.h"

namespace mpk {

#define MPK_GET_VARIANT(I, D, G, N, M) kernel_variant_##I(),
static const KernelVariant* variant_at(int i) {
  static const KernelVariant* const table[kNumVariants] = {MPK_VARIANT_LIST(MPK_GET_VARIANT)};
  return table[i];
}
#undef MPK_GET_VARIANT

static const KernelVariant* pick_variant(uint32_t d, uint32_t grp, uint32_t batch, bool moe, bool large_tasks) {
  const int n = kNumVariants;
  for (int pass = (batch == 1 && large_tasks) ? 0 : 1; pass < 2; ++pass) {
    const int nb = batch == 1 ? (pass == 0 ? 9 : 1) : (batch > 4 && batch <= 16 ? 8 : -1);
    for (int i = 0; i < n; ++i) {
      const KernelVariant* v = variant_at(i);
      if (v->d == (int)d && v->grp == (int)grp && v->nb == nb && v->moe == moe) return v;
    }
  }
  return variant_at(moe ? 7 : 6);   // the generic fallbacks: dense, mixture of experts
}

// Scratch memory of mpk_decode_step_static: part of the library image, one copy per GPU.  In host
// code this name is only a handle for hipGetSymbolAddress; every use of the memory goes through the
// device address that call returns (static_scratch_base below).
static __device__ __align__(256) unsigned char scratch[MPK_STATIC_SCRATCH_BYTES];

// Streaming-speed calibration (option xcd_balance): every workgroup reads its own contiguous slab
// of `slab16` 16-byte words with the access pattern of the linear bodies and records how long it
// took (100 MHz wall clock).  The eight XCDs of the GPU do not stream equally fast.
__global__ void __launch_bounds__(kThreads) stream_probe_kernel(const u32x4* src, size_t slab16, uint64_t* ticks, uint32_t* sink) {
  const u32x4* p = src + (size_t)blockIdx.x * slab16;
  const uint64_t t0 = wall_clock64();
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i < slab16; i += (size_t)kThreads * 8) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (i + (size_t)u * kThreads < slab16) ? ld_stream16(p + i + (size_t)u * kThreads) : u32x4{0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc.x;   // keeps the loads alive
  __syncthreads();
  if (threadIdx.x == 0) ticks[blockIdx.x] = wall_clock64() - t0;
}

// Fills n 32-bit words (counters to zero before a static step; NaN patterns for MPK_DEBUG_POISON).
// A kernel, not a memset node: a caller may be capturing the stream.
__global__ void __launch_bounds__(256) fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// MPK_DEBUG_POISON: the local data share keeps what the last workgroup on the compute unit left in
// it.  A task that reads a word of it that the task has not written (the tail of a staged row, a
// gain past the end of the input) normally finds an old activation there and gets away with it;
// this kernel, launched with the decode kernels' own LDS size on 512 workgroups (two per compute unit of the
// GPU), leaves NaN patterns (as fp32 and as the upper bf16 of a pair) instead.
__global__ void __launch_bounds__(kThreads) lds_poison_kernel(uint32_t words) {
  extern __shared__ __align__(16) uint32_t poison_lds[];
  volatile uint32_t* p = poison_lds;
  for (uint32_t i = threadIdx.x; i < words; i += kThreads) p[i] = 0x7FC00000u;
  __syncthreads();
}

}  // namespace mpk


// =============================================================================== host side
using namespace mpk;

struct mpk_graph {
  HostGraph h;
  bool host_only = true;
  int device = -1;
  // device allocations
  TaskDesc* d_tasks = nullptr;
  EventDesc* d_events = nullptr;
  uint32_t* d_counters = nullptr;
  uint32_t* d_aot_off = nullptr;
  uint32_t* d_aot = nullptr;
  uint32_t* d_op_list = nullptr;
  uint32_t* d_err = nullptr;
  double* d_inv_freq = nullptr;
  uint64_t* d_trace = nullptr;
  GraphConst* d_const = nullptr;
  const KernelVariant* kv = nullptr;
  uint32_t* d_grp = nullptr;
  uint32_t* d_hier = nullptr;
  // just-in-time launch
  uint64_t* d_evq_buf = nullptr;
  uint32_t* d_evq_tail = nullptr;
  uint32_t* d_sched_state = nullptr;
  uint32_t* d_sched_nev = nullptr;
  uint64_t* d_wq_buf = nullptr;
  uint32_t* d_wq_tail = nullptr;
  uint32_t* d_wq_head = nullptr;
  uint32_t n_sched = 0, evq_cap = 1, wq_cap = 1;
  float* d_arena = nullptr;
  std::vector<uint32_t> op_first, op_count;   // per operator: range in op_list
  uint32_t epoch = 0;
  uint64_t timeout_ticks = 0;
  uint32_t step_flags = 0;   // StepArgs::flags of every launch (trace, jitter, no pre-loading)
  bool lost_one = false;     // MPK_DEBUG_LOSE_NOTIFY has had its launch
  // mpk_decode_step_static: descriptors and graph record relocated into the static scratch array
  // (null when the graph is not eligible), and where its pieces sit in the array (bytes)
  TaskDesc* d_tasks_static = nullptr;
  GraphConst* d_const_static = nullptr;
  unsigned char* static_base = nullptr;
  size_t st_counters = 0, st_hier = 0, st_grp = 0, st_arena = 0, st_need = 0;
  const char* static_refusal = "graph was compiled host_only";
  void* launch_out[2] = {nullptr, nullptr};   // host copy of GraphConst::tokens_out / logits_all (source of the async copy)
  const int32_t* page_table = nullptr;        // paged cache: the table the attention tasks read (device)
  struct mpk_server* server = nullptr;        // serving graph: the server attached to it
};

#define HIP_TRY(expr)                                                              \
  do {                                                                             \
    hipError_t _e = (expr);                                                        \
    if (_e != hipSuccess) {                                                        \
      set_error("%s failed: %s", #expr, hipGetErrorString(_e));                    \
      return MPK_ERR_HIP;                                                          \
    }                                                                              \
  } while (0)

static void free_device(mpk_graph* g) {
  if (g->host_only) return;
  (void)hipFree(g->d_tasks); (void)hipFree(g->d_events); (void)hipFree(g->d_counters);
  (void)hipFree(g->d_aot_off); (void)hipFree(g->d_aot); (void)hipFree(g->d_op_list);
  (void)hipFree(g->d_err); (void)hipFree(g->d_arena);
  (void)hipFree(g->d_inv_freq); (void)hipFree(g->d_grp); (void)hipFree(g->d_trace); (void)hipFree(g->d_hier); (void)hipFree(g->d_const);
  (void)hipFree(g->d_evq_buf); (void)hipFree(g->d_evq_tail); (void)hipFree(g->d_sched_state); (void)hipFree(g->d_sched_nev);
  (void)hipFree(g->d_wq_buf); (void)hipFree(g->d_wq_tail); (void)hipFree(g->d_wq_head);
  (void)hipFree(g->d_tasks_static); (void)hipFree(g->d_const_static);
}

// Device address of this GPU's copy of the static scratch array; looked up once per device, with
// that device current.
static mpk_status static_scratch_base(int device, unsigned char** out) {
  static std::mutex mu;
  static unsigned char* base[64] = {};
  if (device < 0 || device >= 64) { set_error("device index %d out of range", device); return MPK_ERR_INVALID_ARG; }
  std::lock_guard<std::mutex> lock(mu);
  if (!base[device]) {
    int cur = -1;
    HIP_TRY(hipGetDevice(&cur));
    if (cur != device) { set_error("device %d is not current (current: %d)", device, cur); return MPK_ERR_INVALID_ARG; }
    unsigned char* p = nullptr;
    HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(mpk::scratch)));
    if (!p) { set_error("hipGetSymbolAddress returned a null address"); return MPK_ERR_HIP; }
    base[device] = p;
  }
  *out = base[device];
  return MPK_OK;
}

static mpk_status resolve_options(const mpk_compile_options* in, mpk_compile_options* out,
                                  int* n_cu) {
  mpk_compile_options o{};
  if (in) {
    if (in->struct_size != sizeof(mpk_compile_options)) {
      set_error("mpk_compile_options.struct_size is %u, expected %zu", in->struct_size, sizeof(mpk_compile_options));
      return MPK_ERR_INVALID_ARG;
    }
    o = *in;
  } else {
    o.struct_size = sizeof(o);
  }
  if (o.launch_mode > MPK_LAUNCH_PER_OP) { set_error("unknown launch_mode %u", o.launch_mode); return MPK_ERR_INVALID_ARG; }
  int cus = 256;
  if (!o.host_only) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t p;
    HIP_TRY(hipGetDeviceProperties(&p, dev));
    cus = p.multiProcessorCount;
  }
  *n_cu = cus;
  if (o.n_sched_wgs >= (uint32_t)cus) { set_error("n_sched_wgs %u leaves no worker", o.n_sched_wgs); return MPK_ERR_INVALID_ARG; }
  if (o.n_workers == 0) o.n_workers = (uint32_t)cus - o.n_sched_wgs;
  if (!o.host_only && o.launch_mode == MPK_LAUNCH_MEGA && o.n_workers + o.n_sched_wgs > (uint32_t)cus) {
    set_error("%u workers + %u scheduler workgroups exceed the %d compute units: the persistent kernel could not be fully resident", o.n_workers, o.n_sched_wgs, cus);
    return MPK_ERR_RESIDENCY;
  }
  if (o.spin_timeout_ms == 0) o.spin_timeout_ms = 2000;
  *out = o;
  return MPK_OK;
}

// Relative streaming speed of the workers by index mod 8, in thousandths of their mean: the median
// of five timed runs of the probe over `bytes` of weights (after one warm-up run).
static mpk_status measure_worker_speeds(const void* weights, size_t bytes, uint32_t n_workers, uint32_t out[8]) {
  const size_t slab16 = std::min<size_t>(bytes / n_workers, (size_t)8 << 20) / 16;
  if (slab16 < 4096) { set_error("xcd_balance: the LM head is too small to time a streaming probe on"); return MPK_ERR_UNSUPPORTED; }
  uint64_t* d_ticks = nullptr;
  uint32_t* d_sink = nullptr;
  if (hipMalloc((void**)&d_ticks, n_workers * sizeof(uint64_t)) != hipSuccess || hipMalloc((void**)&d_sink, 16) != hipSuccess) {
    (void)hipFree(d_ticks);
    set_error("hipMalloc failed for the streaming probe");
    return MPK_ERR_OOM;
  }
  std::vector<uint64_t> t(n_workers);
  std::vector<double> runs[8];
  mpk_status st = MPK_OK;
  for (int rep = 0; rep < 6 && st == MPK_OK; ++rep) {
    hipLaunchKernelGGL(stream_probe_kernel, dim3(n_workers), dim3(kThreads), 0, 0, (const u32x4*)weights, slab16, d_ticks, d_sink);
    if (hipDeviceSynchronize() != hipSuccess || hipMemcpy(t.data(), d_ticks, n_workers * sizeof(uint64_t), hipMemcpyDeviceToHost) != hipSuccess) {
      set_error("streaming probe failed: %s", hipGetErrorString(hipGetLastError()));
      st = MPK_ERR_HIP;
      break;
    }
    if (rep == 0) continue;
    double sum[8] = {0}, n[8] = {0};
    for (uint32_t w = 0; w < n_workers; ++w) { sum[w & 7u] += (double)t[w]; n[w & 7u] += 1.0; }
    for (int k = 0; k < 8; ++k) runs[k].push_back(n[k] > 0 ? sum[k] / n[k] : 0.0);
  }
  (void)hipFree(d_ticks);
  (void)hipFree(d_sink);
  if (st != MPK_OK) return st;
  double speed[8], mean = 0.0;
  int used = 0;
  for (int k = 0; k < 8; ++k) {
    std::sort(runs[k].begin(), runs[k].end());
    const double med = runs[k][runs[k].size() / 2];
    speed[k] = med > 0 ? 1.0 / med : 0.0;
    if (speed[k] > 0) { mean += speed[k]; ++used; }
  }
  mean /= std::max(used, 1);
  for (int k = 0; k < 8; ++k) out[k] = speed[k] > 0 ? (uint32_t)std::lround(1000.0 * speed[k] / mean) : 1000u;
  return MPK_OK;
}

template <typename T>
static mpk_status upload(T** dst, const std::vector<T>& src) {
  size_t bytes = std::max<size_t>(src.size(), 1) * sizeof(T);
  hipError_t e = hipMalloc((void**)dst, bytes);
  if (e != hipSuccess) { set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e)); return MPK_ERR_OOM; }
  if (!src.empty()) HIP_TRY(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
  return MPK_OK;
}

// The dynamic-LDS limit is an attribute of the kernel function, shared by every graph that uses
// the same kernel variant: it is only ever raised, or compiling a graph with a smaller requirement
// would break the launches of an earlier one.
static hipError_t reserve_lds(const void* fn, uint32_t bytes) {
  static std::mutex mu;
  static std::map<const void*, uint32_t> reserved;
  std::lock_guard<std::mutex> lock(mu);
  uint32_t& cur = reserved[fn];
  if (bytes <= cur) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess) cur = bytes;
  return e;
}

extern "C" mpk_status mpk_compile(const mpk_model_config* cfg, const mpk_weight_ptrs* weights,
                                  const mpk_kv_ptrs* kv, const mpk_compile_options* opts,
                                  mpk_graph** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) { set_error("cfg or out is NULL"); return MPK_ERR_INVALID_ARG; }
  mpk_compile_options o;
  int n_cu = 0;
  mpk_status st = resolve_options(opts, &o, &n_cu);
  if (st != MPK_OK) return st;
  if (!o.host_only && o.n_sched_wgs > 0 && !o.force_aot && o.launch_mode != MPK_LAUNCH_MEGA) {
    set_error("scheduler workgroups only exist in the persistent kernel (launch_mode MPK_LAUNCH_MEGA)");
    return MPK_ERR_INVALID_ARG;
  }
  if (o.xcd_balance) {
    if (o.host_only) { set_error("xcd_balance measures on the GPU: not with host_only (set worker_weight_permille instead)"); return MPK_ERR_INVALID_ARG; }
    bool given = false;
    for (int k = 0; k < 8; ++k) given = given || o.worker_weight_permille[k] != 0;
    if (!given && weights && weights->lm_head && cfg->batch <= 4) {
      st = measure_worker_speeds(weights->lm_head, (size_t)cfg->vocab * cfg->hidden * 2, o.n_workers, o.worker_weight_permille);
      if (st != MPK_OK) return st;
    }
  }
  mpk_graph* g = new (std::nothrow) mpk_graph();
  if (!g) { set_error("out of host memory"); return MPK_ERR_OOM; }
  st = build_model_graph(*cfg, weights, kv, o, g->h);
  if (st != MPK_OK) { delete g; return st; }
  g->host_only = o.host_only != 0;
  if (g->host_only) { *out = g; return MPK_OK; }

  auto fail = [&](mpk_status s) { free_device(g); delete g; return s; };
  if (hipGetDevice(&g->device) != hipSuccess) { set_error("hipGetDevice failed"); return fail(MPK_ERR_HIP); }
  HostGraph& h = g->h;
  // residency: dynamic LDS above half of a CU's 160 KB caps occupancy at one workgroup per CU
  // "large": 3 MB or more of weights per worker and layer (8B shape: 1.6 MB, 70B shape: 6.8 MB)
  const bool large_tasks = h.stats.weight_bytes / std::max(1u, cfg->n_layers) / std::max(1u, o.n_workers) >= (3u << 20);
  g->kv = pick_variant(cfg->head_dim, cfg->n_q_heads / cfg->n_kv_heads, cfg->batch, cfg->n_experts != 0, large_tasks);
  hipError_t e = reserve_lds((const void*)g->kv->mega, h.lds_bytes);
  if (e == hipSuccess) e = reserve_lds((const void*)g->kv->op, h.lds_bytes);
  if (e == hipSuccess) e = reserve_lds((const void*)g->kv->loop, h.lds_bytes);
  if (e == hipSuccess) e = reserve_lds((const void*)g->kv->hybrid, h.lds_bytes);
  if (e == hipSuccess && g->kv->run_step) e = reserve_lds((const void*)g->kv->run_step, h.lds_bytes);
  if (e != hipSuccess) { set_error("cannot reserve %u bytes of LDS: %s", h.lds_bytes, hipGetErrorString(e)); return fail(MPK_ERR_RESIDENCY); }
  int per_cu = 0;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)g->kv->mega, kThreads, h.lds_bytes);
  if (e != hipSuccess || per_cu < 1) { set_error("persistent kernel does not fit on a CU (occupancy %d, %s)", per_cu, hipGetErrorString(e)); return fail(MPK_ERR_RESIDENCY); }
  if (o.launch_mode == MPK_LAUNCH_MEGA && (uint64_t)per_cu * n_cu < (uint64_t)o.n_workers + o.n_sched_wgs) {
    set_error("%u workgroups cannot be co-resident on %d CUs x %d", o.n_workers + o.n_sched_wgs, n_cu, per_cu);
    return fail(MPK_ERR_RESIDENCY);
  }
  // activation arena + relocation of the descriptors
  size_t arena_bytes = std::max<size_t>(h.arena_floats, 64) * sizeof(float);
  e = hipMalloc((void**)&g->d_arena, arena_bytes);
  if (e != hipSuccess) { set_error("hipMalloc(%zu) for activations failed: %s", arena_bytes, hipGetErrorString(e)); return fail(MPK_ERR_OOM); }
  if (hipMemset(g->d_arena, 0, arena_bytes) != hipSuccess) { set_error("hipMemset failed"); return fail(MPK_ERR_HIP); }
  std::vector<TaskDesc> descs = h.descs;
  auto reloc = [&](const float* p) -> const float* {
    if (!p) return nullptr;
    return g->d_arena + ((uintptr_t)p / sizeof(float) - 1);
  };
  for (auto& t : descs) {
    t.in = reloc(t.in);
    t.in2 = reloc(t.in2);
    t.out = const_cast<float*>(reloc(t.out));
    if (t.kind == TK_MOE_ROUTE || t.kind == TK_MOE_EXPERT || t.kind == TK_MOE_COMBINE || (t.flags & TF_SPLITK))
      t.aux0 = (void*)reloc((const float*)t.aux0);
  }
  // per-operator task lists (baseline launch mode)
  std::vector<uint32_t> op_list;
  g->op_first.assign(h.ops.size(), 0);
  g->op_count.assign(h.ops.size(), 0);
  {
    std::vector<std::vector<uint32_t>> per(h.ops.size());
    for (uint32_t i = 0; i < h.tasks.size(); ++i)
      if (h.tasks[i].op != MPK_TASK_DUMMY_OP) per[h.tasks[i].op].push_back(i);
    for (size_t oi = 0; oi < per.size(); ++oi) {
      g->op_first[oi] = (uint32_t)op_list.size();
      g->op_count[oi] = (uint32_t)per[oi].size();
      op_list.insert(op_list.end(), per[oi].begin(), per[oi].end());
    }
  }
  std::vector<uint32_t> zeros(h.events.size(), 0), err(8, 0);
  if ((st = upload(&g->d_tasks, descs)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_events, h.events)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_counters, zeros)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_aot_off, h.aot_off)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_aot, h.aot)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_op_list, op_list)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_err, err)) != MPK_OK) return fail(st);
  if ((st = upload(&g->d_inv_freq, h.inv_freq)) != MPK_OK) return fail(st);
  {
    std::vector<uint32_t> gz(h.n_group_counters, 0);
    if ((st = upload(&g->d_grp, gz)) != MPK_OK) return fail(st);
  }
  {
    std::vector<uint32_t> hz((size_t)std::max(h.n_hier_events, 1u) * kHierWordsPerEvent, 0);
    if ((st = upload(&g->d_hier, hz)) != MPK_OK) return fail(st);
  }
  if (o.debug_flags & MPK_DEBUG_TRACE) {
    std::vector<uint64_t> tz(h.tasks.size() * kTraceSlots, 0);
    if ((st = upload(&g->d_trace, tz)) != MPK_OK) return fail(st);
  }
  // just-in-time launch: queues for the scheduler wavefronts (4 per scheduler workgroup)
  {
    const bool jit = o.n_sched_wgs > 0 && !o.force_aot && h.stats.n_jit_tasks > 0;
    g->n_sched = jit ? 4u * o.n_sched_wgs : 0u;
    std::vector<uint32_t> nev(std::max(g->n_sched, 1u), 0);
    uint64_t per_worker = 0;   // bound on the JIT tasks one worker can be handed in a step
    if (jit) {
      for (size_t e = 0; e < h.events.size(); ++e) {
        if (!(h.events[e].flags & EV_JIT)) continue;
        if (e != h.start_event) nev[e % g->n_sched]++;
        per_worker += (h.events[e].last - h.events[e].first + o.n_workers - 1) / o.n_workers;
      }
    }
    auto pow2 = [](uint64_t v) { uint64_t p = 1; while (p < v) p <<= 1; return (uint32_t)p; };
    g->evq_cap = pow2(*std::max_element(nev.begin(), nev.end()) + 1);
    g->wq_cap = pow2(per_worker + 1);
    std::vector<uint64_t> ez((size_t)std::max(g->n_sched, 1u) * g->evq_cap, 0), wz((size_t)o.n_workers * g->wq_cap, 0);
    std::vector<uint32_t> tz((size_t)std::max(g->n_sched, 1u) * 64, 0), wt((size_t)o.n_workers * 64, 0), wh(o.n_workers, 0);
    if ((st = upload(&g->d_evq_buf, ez)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_evq_tail, tz)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_sched_state, tz)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_sched_nev, nev)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_wq_buf, wz)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_wq_tail, wt)) != MPK_OK) return fail(st);
    if ((st = upload(&g->d_wq_head, wh)) != MPK_OK) return fail(st);
  }
  g->timeout_ticks = (uint64_t)o.spin_timeout_ms * 100000ull;   // wall clock counts at 100 MHz
  {
    GraphConst c{};
    c.tasks = g->d_tasks; c.events = g->d_events; c.counters = g->d_counters; c.hier = g->d_hier;
    c.aot_off = g->d_aot_off; c.aot = g->d_aot; c.op_list = g->d_op_list; c.err = g->d_err;
    c.inv_freq = g->d_inv_freq; c.grp_counters = g->d_grp; c.trace = g->d_trace;
    c.timeout_ticks = g->timeout_ticks;
    c.n_workers = h.opt.n_workers;
    c.vocab = h.cfg.vocab; c.max_seq = h.cfg.max_seq; c.n_q = h.cfg.n_q_heads;
    c.n_kv = h.cfg.n_kv_heads; c.head_dim = h.cfg.head_dim; c.batch = h.cfg.batch;
    c.lin_rows_max = h.lin_rows_max; c.lin_res_rows_max = h.lin_res_rows_max; c.lin_page_off = h.lin_page_off;
    c.n_sched = g->n_sched; c.evq_cap = g->evq_cap; c.wq_cap = g->wq_cap;
    c.evq_buf = g->d_evq_buf; c.evq_tail = g->d_evq_tail; c.sched_state = g->d_sched_state;
    c.sched_nev = g->d_sched_nev; c.wq_buf = g->d_wq_buf; c.wq_tail = g->d_wq_tail; c.wq_head = g->d_wq_head;
    c.start_event = h.start_event; c.terminal_event = h.terminal_event;
    c.page_table = nullptr; c.serve = nullptr; c.serve_event = -1;
    c.kv_pages = h.opt.kv_pages;
    for (c.page_shift = 0; h.opt.kv_page_size && (1u << c.page_shift) < h.opt.kv_page_size; ++c.page_shift) {}
    for (const TaskDesc& t : h.descs)
      if (t.kind == TK_SERVE) c.serve_event = t.trig_event;
    std::vector<GraphConst> cv(1, c);
    if ((st = upload(&g->d_const, cv)) != MPK_OK) return fail(st);
    g->step_flags = (g->d_trace ? kTraceBit : 0u) | ((o.debug_flags & MPK_DEBUG_JITTER) ? kJitterBit : 0u) |
                    (o.no_preload ? kNoPreloadBit : 0u);
    // ---- the same graph over the static scratch array (mpk_decode_step_static)
    auto up256 = [](size_t v) { return (v + 255) & ~(size_t)255; };
    g->st_counters = 0;
    g->st_hier = up256(h.events.size() * sizeof(uint32_t));
    g->st_grp = g->st_hier + up256((size_t)std::max(h.n_hier_events, 1u) * kHierWordsPerEvent * sizeof(uint32_t));
    g->st_arena = g->st_grp + up256(std::max<size_t>(h.n_group_counters, 1) * sizeof(uint32_t));
    g->st_need = g->st_arena + up256(arena_bytes);
    g->static_refusal = nullptr;
    if (g->n_sched) g->static_refusal = "graph was compiled with scheduler workgroups";
    else if (h.opt.greedy_loop) g->static_refusal = "graph was compiled with greedy_loop";
    else if (g->d_trace) g->static_refusal = "graph was compiled with MPK_DEBUG_TRACE";
    else if (h.opt.kv_page_size) g->static_refusal = "graph was compiled for a paged KV cache";
    else if (g->st_need > MPK_STATIC_SCRATCH_BYTES) g->static_refusal = "graph needs more scratch memory than the static array holds";
    if (!g->static_refusal) {
      if ((st = static_scratch_base(g->device, &g->static_base)) != MPK_OK) return fail(st);
      float* arena_s = (float*)(g->static_base + g->st_arena);
      std::vector<TaskDesc> ds = h.descs;
      auto reloc_s = [&](const float* p) -> const float* { return p ? arena_s + ((uintptr_t)p / sizeof(float) - 1) : nullptr; };
      for (auto& t : ds) {
        t.in = reloc_s(t.in);
        t.in2 = reloc_s(t.in2);
        t.out = const_cast<float*>(reloc_s(t.out));
        if (t.kind == TK_MOE_ROUTE || t.kind == TK_MOE_EXPERT || t.kind == TK_MOE_COMBINE || (t.flags & TF_SPLITK))
          t.aux0 = (void*)reloc_s((const float*)t.aux0);
      }
      if ((st = upload(&g->d_tasks_static, ds)) != MPK_OK) return fail(st);
      GraphConst cs = c;
      cs.tasks = g->d_tasks_static;
      cs.counters = (uint32_t*)(g->static_base + g->st_counters);
      cs.hier = (uint32_t*)(g->static_base + g->st_hier);
      cs.grp_counters = (uint32_t*)(g->static_base + g->st_grp);
      std::vector<GraphConst> csv(1, cs);
      if ((st = upload(&g->d_const_static, csv)) != MPK_OK) return fail(st);
    }
  }
  *out = g;
  return MPK_OK;
}

extern "C" mpk_status mpk_compile_dag(uint32_t n_tasks, const uint32_t* pairs, size_t n_pairs,
                                      const mpk_compile_options* opts, mpk_graph** out) {
  if (out) *out = nullptr;
  if (!out) { set_error("out is NULL"); return MPK_ERR_INVALID_ARG; }
  mpk_compile_options o{};
  if (opts) {
    if (opts->struct_size != sizeof(mpk_compile_options)) { set_error("bad mpk_compile_options.struct_size"); return MPK_ERR_INVALID_ARG; }
    o = *opts;
  }
  o.host_only = 1;
  if (o.n_workers == 0) o.n_workers = 256 - o.n_sched_wgs;
  mpk_graph* g = new (std::nothrow) mpk_graph();
  if (!g) { set_error("out of host memory"); return MPK_ERR_OOM; }
  mpk_status st = build_dag_graph(n_tasks, pairs, n_pairs, o, g->h);
  if (st != MPK_OK) { delete g; return st; }
  *out = g;
  return MPK_OK;
}

static mpk_status launch_steps(mpk_graph* g, uint32_t n_steps, const int32_t* token_ids, const int32_t* positions,
                               int32_t* tokens_out, float* logits_out, float* logits_all, void* stream,
                               bool static_scratch = false) {
  HostGraph& h = g->h;
  StepArgs a{};
  a.g = (const MPK_CONST GraphConst*)g->d_const;
  a.tasks = g->d_tasks; a.events = g->d_events; a.counters = g->d_counters; a.hier = g->d_hier;
  a.n_sched = g->n_sched; a.flags = g->step_flags;
  if ((h.opt.debug_flags & MPK_DEBUG_LOSE_NOTIFY) && !g->lost_one && h.opt.launch_mode == MPK_LAUNCH_MEGA) {
    a.flags |= kLoseNotifyBit;   // once
    g->lost_one = true;
  }
  a.token_ids = token_ids; a.positions = positions; a.logits = logits_out;
  hipStream_t s = (hipStream_t)stream;
  float* arena = g->d_arena;
  const size_t arena_words = std::max<size_t>(h.arena_floats, 64);
  if (static_scratch) {
    // the step's working memory is the static array: counters start from zero every time (the
    // array is shared by all graphs on this GPU), so this is always "step one"
    a.g = (const MPK_CONST GraphConst*)g->d_const_static;
    a.tasks = g->d_tasks_static;
    a.counters = (uint32_t*)(g->static_base + g->st_counters);
    a.hier = (uint32_t*)(g->static_base + g->st_hier);
    arena = (float*)(g->static_base + g->st_arena);
    hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(256), 0, s, (uint32_t*)g->static_base, g->st_arena / sizeof(uint32_t), 0u);
    HIP_TRY(hipGetLastError());
  }
  if (h.opt.debug_flags & MPK_DEBUG_POISON) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(256), dim3(256), 0, s, (uint32_t*)arena, arena_words, 0x7FC00000u);
    HIP_TRY(hipGetLastError());
    HIP_TRY(reserve_lds((const void*)lds_poison_kernel, h.lds_bytes));
    hipLaunchKernelGGL(lds_poison_kernel, dim3(512), dim3(kThreads), h.lds_bytes, s, h.lds_bytes / 4u);
    HIP_TRY(hipGetLastError());
  }
  if (h.opt.launch_mode == MPK_LAUNCH_MEGA) {
    // events compare their counters with the step number, a launch argument: a captured launch
    // replayed later would carry a stale one and wait for nothing
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (s != nullptr && hipStreamIsCapturing(s, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
      set_error("a persistent-kernel launch cannot be captured into a HIP graph");
      return MPK_ERR_UNSUPPORTED;
    }
  }
  if (h.opt.greedy_loop) {   // output pointers of this launch -> graph record, ordered on the stream
    g->launch_out[0] = tokens_out; g->launch_out[1] = logits_all;
    HIP_TRY(hipMemcpyAsync((char*)g->d_const + offsetof(GraphConst, tokens_out), g->launch_out, sizeof(g->launch_out),
                           hipMemcpyHostToDevice, s));
  }
  if (h.opt.launch_mode == MPK_LAUNCH_MEGA) {
    a.epoch = static_scratch ? 1u : g->epoch + 1;
    a.step = 0; a.n_steps = (uint16_t)n_steps;
    if (!static_scratch) g->epoch += n_steps;
    // Several steps: one launch of the loop kernel -- or, where the kernel set has a single-step
    // kernel for runs (every set compiled for a model shape), a launch of that kernel per step, back
    // to back with no host synchronisation: inside the step loop the linear bodies come out slower
    // (8B shape, batch 1: 3.12 against 3.01 ms per token; batch 8: 4.93 against 4.87), and the GPU
    // front end overlaps back-to-back launches almost completely.  greedy_loop = 2 asks for the
    // single launch regardless.
    const bool by_step = n_steps > 1 && h.opt.greedy_loop != 2 && !g->n_sched && g->kv->run_step != nullptr;
    if (by_step || n_steps == 1) a.flags |= kOneStepBit;
    if (by_step) {
      for (uint32_t i = 0; i < n_steps; ++i) {
        a.step = (uint16_t)i;
        hipLaunchKernelGGL(g->kv->run_step, dim3(h.opt.n_workers), dim3(kThreads), h.lds_bytes, s, a);
        ++a.epoch;
      }
    } else if (n_steps > 1)   // (callers have checked: no scheduler workgroups)
      hipLaunchKernelGGL(g->kv->loop, dim3(h.opt.n_workers), dim3(kThreads), h.lds_bytes, s, a);
    else if (g->n_sched)
      hipLaunchKernelGGL(g->kv->hybrid, dim3(h.opt.n_workers + h.opt.n_sched_wgs), dim3(kThreads), h.lds_bytes, s, a);
    else
      hipLaunchKernelGGL(g->kv->mega, dim3(h.opt.n_workers), dim3(kThreads), h.lds_bytes, s, a);
    HIP_TRY(hipGetLastError());
  } else {
    a.n_steps = (uint16_t)n_steps;
    for (uint32_t step = 0; step < n_steps; ++step) {
      a.epoch = static_scratch ? 1u : ++g->epoch;
      a.step = (uint16_t)step;
      for (size_t oi = 0; oi < h.ops.size(); ++oi) {
        if (!g->op_count[oi]) continue;
        hipLaunchKernelGGL(g->kv->op, dim3(g->op_count[oi]), dim3(kThreads), h.lds_bytes, s, a,
                           g->op_first[oi]);
      }
    }
    HIP_TRY(hipGetLastError());
  }
  return MPK_OK;
}

extern "C" mpk_status mpk_decode_step(mpk_graph* g, const int32_t* token_ids,
                                      const int32_t* positions, float* logits_out, void* stream) {
  if (!g || !token_ids || !positions || !logits_out) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only) { set_error("graph was compiled host_only"); return MPK_ERR_INVALID_ARG; }
  if (g->h.opt.greedy_loop) { set_error("graph was compiled with greedy_loop: it samples and advances tokens and positions itself, run it with mpk_decode_steps"); return MPK_ERR_INVALID_ARG; }
  if (g->h.opt.kv_page_size && !g->page_table) { set_error("the graph reads a paged KV cache: give it a page table first (mpk_graph_set_page_table)"); return MPK_ERR_INVALID_ARG; }
  return launch_steps(g, 1, token_ids, positions, nullptr, logits_out, nullptr, stream);
}

extern "C" mpk_status mpk_decode_step_static(mpk_graph* g, const int32_t* token_ids, const int32_t* positions,
                                             float* logits_out, void* stream) {
  if (!g || !token_ids || !positions || !logits_out) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (g->static_refusal) {
    set_error("mpk_decode_step_static: %s (needs %zu bytes, the array holds %u)", g->static_refusal, g->st_need, (unsigned)MPK_STATIC_SCRATCH_BYTES);
    return g->host_only ? MPK_ERR_INVALID_ARG : MPK_ERR_UNSUPPORTED;
  }
  int cur = -1;
  HIP_TRY(hipGetDevice(&cur));
  if (cur != g->device) { set_error("the graph lives on device %d, device %d is current", g->device, cur); return MPK_ERR_INVALID_ARG; }
  return launch_steps(g, 1, token_ids, positions, nullptr, logits_out, nullptr, stream, true);
}

extern "C" size_t mpk_static_scratch_need(const mpk_graph* g) { return (g && !g->host_only) ? g->st_need : 0; }

extern "C" mpk_status mpk_decode_steps(mpk_graph* g, uint32_t n_steps, int32_t* token_ids, int32_t* positions,
                                       int32_t* tokens_out, float* logits_out, float* logits_all, void* stream) {
  if (!g || !token_ids || !positions || !logits_out) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only) { set_error("graph was compiled host_only"); return MPK_ERR_INVALID_ARG; }
  if (!g->h.opt.greedy_loop) { set_error("mpk_decode_steps needs a graph compiled with greedy_loop = 1"); return MPK_ERR_INVALID_ARG; }
  if (n_steps == 0 || n_steps > g->h.cfg.max_seq || n_steps > 65535u) { set_error("n_steps %u out of range (1..min(max_seq, 65535))", n_steps); return MPK_ERR_INVALID_ARG; }
  if (g->n_sched && n_steps > 1) { set_error("several steps per launch are only supported without scheduler workgroups"); return MPK_ERR_UNSUPPORTED; }
  if (g->h.opt.serving) { set_error("a serving graph is run through its server (mpk_serve_run)"); return MPK_ERR_INVALID_ARG; }
  if (g->h.opt.kv_page_size && !g->page_table) { set_error("the graph reads a paged KV cache: give it a page table first (mpk_graph_set_page_table)"); return MPK_ERR_INVALID_ARG; }
  return launch_steps(g, n_steps, token_ids, positions, tokens_out, logits_out, logits_all, stream);
}

extern "C" mpk_status mpk_graph_status(mpk_graph* g) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only) return MPK_OK;
  uint32_t err[4] = {0, 0, 0, 0};
  HIP_TRY(hipMemcpy(err, g->d_err, sizeof(err), hipMemcpyDeviceToHost));
  switch (err[0]) {
    case DE_NONE: return MPK_OK;
    case DE_TIMEOUT:
      set_error("watchdog: worker %u waited too long on event %u; call mpk_graph_reset", err[3], err[2]);
      return MPK_ERR_TIMEOUT;
    case DE_BAD_POSITION:
      set_error("sequence %u has position %d outside [0, max_seq)", err[2], (int)err[3]);
      return MPK_ERR_DEVICE;
    case DE_BAD_TOKEN:
      set_error("sequence %u has token %d outside [0, vocab)", err[2], (int)err[3]);
      return MPK_ERR_DEVICE;
    case DE_BAD_PAGE:
      set_error("sequence %u: a page-table entry for rows from %u on is outside the pool", err[2], err[3]);
      return MPK_ERR_DEVICE;
    case DE_BAD_META:
      set_error("an expert task found an inconsistent meta-tensor (expert %u, %u tokens)", err[2], err[3]);
      return MPK_ERR_DEVICE;
    default: set_error("unknown device error %u", err[0]); return MPK_ERR_DEVICE;
  }
}

static hipError_t server_forget_drained(mpk_server* s);

extern "C" mpk_status mpk_graph_reset(mpk_graph* g) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only) return MPK_OK;
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemset(g->d_counters, 0, g->h.events.size() * sizeof(uint32_t)));
  HIP_TRY(hipMemset(g->d_err, 0, 8 * sizeof(uint32_t)));
  HIP_TRY(hipMemset(g->d_hier, 0, (size_t)std::max(g->h.n_hier_events, 1u) * kHierWordsPerEvent * sizeof(uint32_t)));
  HIP_TRY(hipMemset(g->d_grp, 0, std::max<size_t>(g->h.n_group_counters, 1) * sizeof(uint32_t)));
  if (g->server) HIP_TRY(server_forget_drained(g->server));   // (step numbers start over)
  {
    const size_t ns = std::max(g->n_sched, 1u), nw = g->h.opt.n_workers;
    HIP_TRY(hipMemset(g->d_evq_buf, 0, ns * g->evq_cap * sizeof(uint64_t)));
    HIP_TRY(hipMemset(g->d_evq_tail, 0, ns * 64 * sizeof(uint32_t)));
    HIP_TRY(hipMemset(g->d_sched_state, 0, ns * 64 * sizeof(uint32_t)));
    HIP_TRY(hipMemset(g->d_wq_buf, 0, nw * g->wq_cap * sizeof(uint64_t)));
    HIP_TRY(hipMemset(g->d_wq_tail, 0, nw * 64 * sizeof(uint32_t)));
    HIP_TRY(hipMemset(g->d_wq_head, 0, nw * sizeof(uint32_t)));
  }
  HIP_TRY(hipDeviceSynchronize());
  g->epoch = 0;
  return MPK_OK;
}

extern "C" mpk_status mpk_graph_stats(const mpk_graph* g, mpk_stats* out) {
  if (!g || !out) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  *out = g->h.stats;
  out->struct_size = sizeof(mpk_stats);
  return MPK_OK;
}

extern "C" mpk_status mpk_graph_export(const mpk_graph* g, void* buf, size_t cap, size_t* need) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  size_t n = export_size(g->h);
  if (need) *need = n;
  if (!buf) return MPK_OK;
  if (cap < n) { set_error("export buffer too small: %zu < %zu", cap, n); return MPK_ERR_INVALID_ARG; }
  export_graph(g->h, buf);
  return MPK_OK;
}

extern "C" mpk_status mpk_graph_trace(mpk_graph* g, uint64_t* buf, size_t cap, size_t* need) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only || !g->d_trace) { set_error("graph was not compiled with MPK_DEBUG_TRACE"); return MPK_ERR_INVALID_ARG; }
  size_t n = g->h.tasks.size() * kTraceSlots;
  if (need) *need = n;
  if (!buf) return MPK_OK;
  if (cap < n) { set_error("trace buffer too small: %zu < %zu", cap, n); return MPK_ERR_INVALID_ARG; }
  HIP_TRY(hipMemcpy(buf, g->d_trace, n * sizeof(uint64_t), hipMemcpyDeviceToHost));
  return MPK_OK;
}

extern "C" mpk_status mpk_graph_moe_active(mpk_graph* g, uint32_t* out, size_t cap, size_t* need) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only || g->h.moe_meta_offset.empty()) { set_error("not a mixture-of-experts graph on a device"); return MPK_ERR_INVALID_ARG; }
  const size_t n = g->h.moe_meta_offset.size();
  if (need) *need = n;
  if (!out) return MPK_OK;
  if (cap < n) { set_error("buffer too small: %zu < %zu", cap, n); return MPK_ERR_INVALID_ARG; }
  for (size_t l = 0; l < n; ++l)
    HIP_TRY(hipMemcpy(out + l, g->d_arena + g->h.moe_meta_offset[l], sizeof(uint32_t), hipMemcpyDeviceToHost));
  return MPK_OK;
}

extern "C" mpk_status mpk_graph_moe_selection(mpk_graph* g, uint32_t* experts, float* weights, size_t cap, size_t* need) {
  if (!g) { set_error("NULL graph"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only || g->h.moe_meta_offset.empty()) { set_error("not a mixture-of-experts graph on a device"); return MPK_ERR_INVALID_ARG; }
  const size_t L = g->h.moe_meta_offset.size(), E = g->h.cfg.n_experts, P = (size_t)g->h.cfg.batch * g->h.cfg.top_k;
  if (need) *need = L * P;
  if (!experts && !weights) return MPK_OK;
  if (cap < L * P) { set_error("buffer too small: %zu < %zu", cap, L * P); return MPK_ERR_INVALID_ARG; }
  for (size_t l = 0; l < L; ++l) {
    const float* meta = g->d_arena + g->h.moe_meta_offset[l];
    if (weights) HIP_TRY(hipMemcpy(weights + l * P, meta + 2 + 3 * E + P, P * sizeof(float), hipMemcpyDeviceToHost));
    if (experts) HIP_TRY(hipMemcpy(experts + l * P, meta + 2 + 3 * E + 2 * P, P * sizeof(uint32_t), hipMemcpyDeviceToHost));
  }
  return MPK_OK;
}

// ------------------------------------------------------------------------------ graph sets
// Section 6.1 ("Supporting runtime dynamism"): one task graph per representative batch size, the
// powers of two up to the maximum; the smallest that holds the active sequences runs.
struct mpk_graph_set {
  std::vector<mpk_graph*> graphs;   // ascending batch size; the last one is the maximum batch
  std::vector<uint32_t> batch;
};

extern "C" void mpk_set_destroy(mpk_graph_set* s) {
  if (!s) return;
  for (mpk_graph* g : s->graphs) mpk_graph_destroy(g);
  delete s;
}

extern "C" mpk_status mpk_compile_set(const mpk_model_config* cfg, const mpk_weight_ptrs* weights,
                                      const mpk_kv_ptrs* kv, const mpk_compile_options* opts,
                                      mpk_graph_set** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) { set_error("cfg or out is NULL"); return MPK_ERR_INVALID_ARG; }
  if (cfg->struct_size != sizeof(mpk_model_config)) { set_error("mpk_model_config.struct_size is %u, expected %zu", cfg->struct_size, sizeof(mpk_model_config)); return MPK_ERR_INVALID_ARG; }
  if (cfg->batch == 0) { set_error("a model dimension is zero"); return MPK_ERR_INVALID_ARG; }
  mpk_compile_options o{};
  if (opts) {
    if (opts->struct_size != sizeof(mpk_compile_options)) {
      set_error("mpk_compile_options.struct_size is %u, expected %zu", opts->struct_size, sizeof(mpk_compile_options));
      return MPK_ERR_INVALID_ARG;
    }
    o = *opts;
  } else {
    o.struct_size = sizeof(o);
  }
  if (o.kv_batch != 0) { set_error("kv_batch is set by mpk_compile_set itself"); return MPK_ERR_INVALID_ARG; }
  if (!o.kv_page_size) o.kv_batch = cfg->batch;   // (a paged pool has no batch extent: every graph reads it through its table)
  mpk_graph_set* s = new (std::nothrow) mpk_graph_set();
  if (!s) { set_error("out of host memory"); return MPK_ERR_OOM; }
  std::vector<uint32_t> sizes;
  for (uint32_t b = 1; b < cfg->batch; b *= 2) sizes.push_back(b);
  sizes.push_back(cfg->batch);
  for (uint32_t b : sizes) {
    mpk_model_config c = *cfg;
    c.batch = b;
    mpk_graph* g = nullptr;
    const mpk_status st = mpk_compile(&c, weights, kv, &o, &g);
    if (st != MPK_OK) { mpk_set_destroy(s); return st; }   // (the message of the failed compile stands)
    s->graphs.push_back(g);
    s->batch.push_back(b);
  }
  *out = s;
  return MPK_OK;
}

extern "C" uint32_t mpk_set_size(const mpk_graph_set* s) { return s ? (uint32_t)s->graphs.size() : 0u; }

extern "C" mpk_graph* mpk_set_graph(mpk_graph_set* s, uint32_t i) {
  return (s && i < s->graphs.size()) ? s->graphs[i] : nullptr;
}

extern "C" uint32_t mpk_set_batch_for(const mpk_graph_set* s, uint32_t n_active) {
  if (!s || n_active == 0) return 0;
  for (uint32_t b : s->batch)
    if (b >= n_active) return b;
  return 0;
}

extern "C" mpk_status mpk_set_decode_step(mpk_graph_set* s, uint32_t n_active, const int32_t* token_ids,
                                          const int32_t* positions, float* logits_out, void* stream) {
  if (!s) { set_error("set is NULL"); return MPK_ERR_INVALID_ARG; }
  for (size_t i = 0; i < s->graphs.size(); ++i)
    if (n_active != 0 && s->batch[i] >= n_active) return mpk_decode_step(s->graphs[i], token_ids, positions, logits_out, stream);
  set_error("n_active %u is outside 1..%u", n_active, s->batch.empty() ? 0u : s->batch.back());
  return MPK_ERR_INVALID_ARG;
}

// ------------------------------------------------------------------ paged cache and serving
extern "C" mpk_status mpk_graph_set_page_table(mpk_graph* g, const int32_t* page_table) {
  if (!g || !page_table) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (g->host_only) { set_error("graph was compiled host_only"); return MPK_ERR_INVALID_ARG; }
  if (!g->h.opt.kv_page_size) { set_error("the graph was compiled for a contiguous KV cache"); return MPK_ERR_INVALID_ARG; }
  if (g->h.opt.serving) { set_error("a serving graph's page table belongs to its server"); return MPK_ERR_INVALID_ARG; }
  HIP_TRY(hipMemcpy((char*)g->d_const + offsetof(GraphConst, page_table), &page_table, sizeof(page_table), hipMemcpyHostToDevice));
  g->page_table = page_table;
  return MPK_OK;
}

struct mpk_server {
  mpk_graph* g = nullptr;              // the graph of the largest batch size
  std::vector<mpk_graph*> graphs;      // ascending batch size (one entry unless created over a graph set)
  mpk_serve_config cfg{};
  uint32_t batch = 0, max_blocks = 0, n_submitted = 0;
  uint32_t known_done = 0;             // requests known to have finished (read back by mpk_serve_state / _result)
  uint32_t last_batch = 0;             // batch size of the graph the last launch ran on
  // device state (ServeDev points into these)
  int32_t *d_slot = nullptr, *d_table = nullptr, *d_free = nullptr, *d_prompt = nullptr, *d_out = nullptr;
  int32_t *d_tokens = nullptr, *d_positions = nullptr;
  uint32_t *d_scalars = nullptr, *d_len = nullptr, *d_state = nullptr;
  float* d_logits = nullptr;
  ServeDev* d_rec = nullptr;
  // host staging that outlives the asynchronous copies of mpk_serve_submit
  std::vector<std::vector<int32_t>> prompts;
  std::vector<uint32_t> lens, tails;
};

static hipError_t server_forget_drained(mpk_server* s) { return hipMemset(s->d_scalars + kServeStop, 0, sizeof(uint32_t)); }

static void server_free(mpk_server* s) {
  (void)hipFree(s->d_slot); (void)hipFree(s->d_table); (void)hipFree(s->d_free); (void)hipFree(s->d_prompt);
  (void)hipFree(s->d_out); (void)hipFree(s->d_tokens); (void)hipFree(s->d_positions); (void)hipFree(s->d_scalars);
  (void)hipFree(s->d_len); (void)hipFree(s->d_state); (void)hipFree(s->d_logits); (void)hipFree(s->d_rec);
}

static mpk_status serve_create(const std::vector<mpk_graph*>& graphs, const mpk_serve_config* cfg, mpk_server** out) {
  if (out) *out = nullptr;
  if (graphs.empty() || !graphs.back() || !cfg || !out) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (cfg->struct_size != sizeof(mpk_serve_config)) { set_error("mpk_serve_config.struct_size is %u, expected %zu", cfg->struct_size, sizeof(mpk_serve_config)); return MPK_ERR_INVALID_ARG; }
  mpk_graph* g = graphs.back();
  for (mpk_graph* x : graphs) {
    if (x->host_only || !x->h.opt.serving) { set_error("the graph was not compiled with serving = 1 (or is host_only)"); return MPK_ERR_INVALID_ARG; }
    if (x->server) { set_error("the graph already has a server"); return MPK_ERR_INVALID_ARG; }
    if (x->h.opt.kv_page_size != g->h.opt.kv_page_size || x->h.opt.kv_pages != g->h.opt.kv_pages || x->device != g->device ||
        x->h.cfg.max_seq != g->h.cfg.max_seq || x->h.cfg.vocab != g->h.cfg.vocab || x->h.cfg.batch > g->h.cfg.batch) {
      set_error("the graphs of a served set must share the paged cache, max_seq and vocab");
      return MPK_ERR_INVALID_ARG;
    }
  }
  const mpk_model_config& c = g->h.cfg;
  if (g->h.opt.kv_pages <= c.batch) { set_error("kv_pages %u: the pool needs more pages than the %u batch slots", g->h.opt.kv_pages, c.batch); return MPK_ERR_INVALID_ARG; }
  const uint32_t ps = g->h.opt.kv_page_size, n_pages = g->h.opt.kv_pages, B = c.batch;
  if (!cfg->max_requests || !cfg->max_prompt || !cfg->max_new || cfg->max_prompt > c.max_seq || cfg->max_new > c.max_seq ||
      cfg->max_requests > (1u << 20)) {
    set_error("mpk_serve_config: max_requests (1..2^20), max_prompt and max_new (1..max_seq) out of range");
    return MPK_ERR_INVALID_ARG;
  }
  int cur = -1;
  HIP_TRY(hipGetDevice(&cur));
  if (cur != g->device) { set_error("the graph lives on device %d, device %d is current", g->device, cur); return MPK_ERR_INVALID_ARG; }
  mpk_server* s = new (std::nothrow) mpk_server();
  if (!s) { set_error("out of host memory"); return MPK_ERR_OOM; }
  s->g = g; s->graphs = graphs; s->cfg = *cfg; s->batch = B; s->max_blocks = c.max_seq / ps;
  auto fail = [&](mpk_status st) { server_free(s); delete s; return st; };
  // initial state: every slot idle in its own page, every other page free (lowest number on top)
  std::vector<int32_t> slot(3 * (size_t)B, 0), table((size_t)B * s->max_blocks, -1), free_stack(n_pages, -1), zb(B, 0);
  for (uint32_t b = 0; b < B; ++b) { slot[b] = -1; table[(size_t)b * s->max_blocks] = (int32_t)b; }
  for (uint32_t i = 0; i + B < n_pages; ++i) free_stack[i] = (int32_t)(n_pages - 1 - i);
  std::vector<uint32_t> scalars(kServeScalars, 0);
  scalars[kServeNFree] = n_pages - B;
  std::vector<int32_t> prompt0((size_t)cfg->max_requests * cfg->max_prompt, 0), out0((size_t)cfg->max_requests * cfg->max_new, -1);
  std::vector<uint32_t> len0(2 * (size_t)cfg->max_requests, 0);
  std::vector<float> lg((size_t)B * c.vocab, 0.f);
  mpk_status st;
  if ((st = upload(&s->d_slot, slot)) != MPK_OK || (st = upload(&s->d_table, table)) != MPK_OK ||
      (st = upload(&s->d_free, free_stack)) != MPK_OK || (st = upload(&s->d_scalars, scalars)) != MPK_OK ||
      (st = upload(&s->d_prompt, prompt0)) != MPK_OK || (st = upload(&s->d_out, out0)) != MPK_OK ||
      (st = upload(&s->d_len, len0)) != MPK_OK || (st = upload(&s->d_state, len0)) != MPK_OK ||
      (st = upload(&s->d_tokens, zb)) != MPK_OK || (st = upload(&s->d_positions, zb)) != MPK_OK ||
      (st = upload(&s->d_logits, lg)) != MPK_OK)
    return fail(st);
  ServeDev rec{};
  rec.slot_req = s->d_slot; rec.slot_pos = s->d_slot + B; rec.slot_held = s->d_slot + 2 * B;
  rec.table = s->d_table; rec.free_stack = s->d_free; rec.scalars = s->d_scalars;
  rec.req_prompt = s->d_prompt; rec.req_len = s->d_len; rec.req_out = s->d_out; rec.req_state = s->d_state;
  rec.max_blocks = s->max_blocks; rec.max_prompt = cfg->max_prompt; rec.max_new = cfg->max_new;
  rec.max_requests = cfg->max_requests; rec.eos = cfg->eos_token;
  for (rec.page_shift = 0; (1u << rec.page_shift) < ps; ++rec.page_shift) {}
  std::vector<ServeDev> rv(1, rec);
  if ((st = upload(&s->d_rec, rv)) != MPK_OK) return fail(st);
  const void* ptrs[2] = {s->d_table, s->d_rec};
  static_assert(offsetof(GraphConst, serve) == offsetof(GraphConst, page_table) + sizeof(void*), "page_table and serve are adjacent");
  for (mpk_graph* x : graphs)
    if (hipMemcpy((char*)x->d_const + offsetof(GraphConst, page_table), ptrs, sizeof(ptrs), hipMemcpyHostToDevice) != hipSuccess) {
      set_error("hipMemcpy of the serving record failed");
      return fail(MPK_ERR_HIP);
    }
  s->lens.reserve(2 * (size_t)cfg->max_requests);
  s->tails.reserve(cfg->max_requests);
  for (mpk_graph* x : graphs) {
    x->page_table = s->d_table;
    x->server = s;
  }
  *out = s;
  return MPK_OK;
}

extern "C" mpk_status mpk_serve_create(mpk_graph* g, const mpk_serve_config* cfg, mpk_server** out) {
  if (out) *out = nullptr;
  if (!g) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  return serve_create(std::vector<mpk_graph*>(1, g), cfg, out);
}

extern "C" mpk_status mpk_serve_create_set(mpk_graph_set* set, const mpk_serve_config* cfg, mpk_server** out) {
  if (out) *out = nullptr;
  if (!set || set->graphs.empty()) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  return serve_create(set->graphs, cfg, out);
}

extern "C" uint32_t mpk_serve_last_batch(const mpk_server* s) { return s ? s->last_batch : 0u; }

extern "C" mpk_status mpk_serve_status(mpk_server* s) {
  if (!s) { set_error("NULL server"); return MPK_ERR_INVALID_ARG; }
  for (mpk_graph* x : s->graphs) {
    const mpk_status st = mpk_graph_status(x);
    if (st != MPK_OK) return st;
  }
  return MPK_OK;
}

extern "C" mpk_status mpk_serve_submit(mpk_server* s, const int32_t* prompt, uint32_t prompt_len, uint32_t max_new_tokens,
                                       void* stream, uint32_t* request_id) {
  if (!s || !prompt) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  const mpk_model_config& c = s->g->h.cfg;
  const uint32_t ps = s->g->h.opt.kv_page_size;
  if (s->n_submitted >= s->cfg.max_requests) { set_error("the server has taken its max_requests = %u requests", s->cfg.max_requests); return MPK_ERR_UNSUPPORTED; }
  if (prompt_len == 0 || prompt_len > s->cfg.max_prompt || max_new_tokens == 0 || max_new_tokens > s->cfg.max_new) {
    set_error("prompt_len %u (1..%u) or max_new_tokens %u (1..%u) out of range", prompt_len, s->cfg.max_prompt, max_new_tokens, s->cfg.max_new);
    return MPK_ERR_INVALID_ARG;
  }
  const uint64_t rows = (uint64_t)prompt_len + max_new_tokens - 1;
  if (rows > c.max_seq) { set_error("the request would cache %llu rows, max_seq is %u", (unsigned long long)rows, c.max_seq); return MPK_ERR_INVALID_ARG; }
  if ((rows + ps - 1) / ps > s->g->h.opt.kv_pages - c.batch) { set_error("the request needs more pages than the pool can ever free"); return MPK_ERR_INVALID_ARG; }
  for (uint32_t i = 0; i < prompt_len; ++i)
    if (prompt[i] < 0 || (uint32_t)prompt[i] >= c.vocab) { set_error("prompt token %u is %d, outside [0, vocab)", i, prompt[i]); return MPK_ERR_INVALID_ARG; }
  const uint32_t r = s->n_submitted;
  s->prompts.emplace_back(prompt, prompt + prompt_len);
  s->lens.push_back(prompt_len); s->lens.push_back(max_new_tokens);
  s->tails.push_back(r + 1);
  hipStream_t st = (hipStream_t)stream;
  HIP_TRY(hipMemcpyAsync(s->d_prompt + (size_t)r * s->cfg.max_prompt, s->prompts.back().data(), prompt_len * sizeof(int32_t), hipMemcpyHostToDevice, st));
  HIP_TRY(hipMemcpyAsync(s->d_len + 2 * (size_t)r, &s->lens[2 * (size_t)r], 2 * sizeof(uint32_t), hipMemcpyHostToDevice, st));
  // the queue's tail last: a request is visible to the serving task only with its prompt in place
  HIP_TRY(hipMemcpyAsync(s->d_scalars + kServeQTail, &s->tails[r], sizeof(uint32_t), hipMemcpyHostToDevice, st));
  s->n_submitted = r + 1;
  if (request_id) *request_id = r;
  return MPK_OK;
}

extern "C" mpk_status mpk_serve_run(mpk_server* s, uint32_t n_iterations, void* stream) {
  if (!s) { set_error("NULL server"); return MPK_ERR_INVALID_ARG; }
  if (n_iterations == 0 || n_iterations > 65535u) { set_error("n_iterations %u out of range (1..65535)", n_iterations); return MPK_ERR_INVALID_ARG; }
  // Section 6.1: the task graph specialised for the smallest batch size that holds the current
  // batch.  The running requests always fill the lowest slots (the serving task closes ranks), and
  // there are at most (submitted - finished) of them plus arrivals; "finished" is what the host has
  // read back so far, so the bound errs on the large side.
  const uint32_t open = std::max(1u, std::min(s->batch, s->n_submitted - std::min(s->known_done, s->n_submitted)));
  mpk_graph* g = s->g;
  for (mpk_graph* x : s->graphs)
    if (x->h.cfg.batch >= open) { g = x; break; }
  s->last_batch = g->h.cfg.batch;
  // the "drained" marker is a step number of the graph that ran: each graph of a set counts its
  // own steps, so the marker starts every launch at zero (no step has that number)
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, s->d_scalars + kServeStop, (size_t)1, 0u);
  HIP_TRY(hipGetLastError());
  const uint32_t keep = g->step_flags;
  g->step_flags |= kServeBit;
  const mpk_status st = launch_steps(g, n_iterations, s->d_tokens, s->d_positions, nullptr, s->d_logits, nullptr, stream);
  g->step_flags = keep;
  return st;
}

extern "C" mpk_status mpk_serve_result(mpk_server* s, uint32_t request_id, int32_t* tokens, size_t cap, uint32_t* n_tokens,
                                       uint32_t* state) {
  if (!s || !n_tokens || !state) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  if (request_id >= s->n_submitted) { set_error("request %u was never submitted", request_id); return MPK_ERR_INVALID_ARG; }
  uint32_t st[2] = {0, 0};
  HIP_TRY(hipMemcpy(st, s->d_state + 2 * (size_t)request_id, sizeof(st), hipMemcpyDeviceToHost));
  *state = st[0];
  *n_tokens = st[1];
  HIP_TRY(hipMemcpy(&s->known_done, s->d_scalars + kServeDone, sizeof(uint32_t), hipMemcpyDeviceToHost));
  const size_t n = std::min<size_t>(st[1], cap);
  if (n && tokens) HIP_TRY(hipMemcpy(tokens, s->d_out + (size_t)request_id * s->cfg.max_new, n * sizeof(int32_t), hipMemcpyDeviceToHost));
  return MPK_OK;
}

extern "C" mpk_status mpk_serve_state(mpk_server* s, int32_t* buf, size_t cap, size_t* need) {
  if (!s || !need) { set_error("NULL argument"); return MPK_ERR_INVALID_ARG; }
  const uint32_t B = s->batch, mb = s->max_blocks, n_pages = s->g->h.opt.kv_pages;
  const size_t n = 8 + 5 * (size_t)B + (size_t)B * mb + n_pages;
  *need = n;
  if (!buf || cap < n) return MPK_OK;
  uint32_t sc[kServeScalars];
  HIP_TRY(hipMemcpy(sc, s->d_scalars, sizeof(sc), hipMemcpyDeviceToHost));
  buf[0] = (int32_t)B; buf[1] = (int32_t)mb; buf[2] = (int32_t)sc[kServeNFree]; buf[3] = (int32_t)sc[kServePromised];
  buf[4] = (int32_t)sc[kServeQHead]; buf[5] = (int32_t)sc[kServeQTail]; buf[6] = (int32_t)sc[kServeIterations]; buf[7] = (int32_t)sc[kServeTokens];
  s->known_done = sc[kServeDone];
  int32_t* p = buf + 8;
  HIP_TRY(hipMemcpy(p, s->d_slot, 3 * (size_t)B * sizeof(int32_t), hipMemcpyDeviceToHost)); p += 3 * (size_t)B;
  HIP_TRY(hipMemcpy(p, s->d_tokens, B * sizeof(int32_t), hipMemcpyDeviceToHost)); p += B;
  HIP_TRY(hipMemcpy(p, s->d_positions, B * sizeof(int32_t), hipMemcpyDeviceToHost)); p += B;
  HIP_TRY(hipMemcpy(p, s->d_table, (size_t)B * mb * sizeof(int32_t), hipMemcpyDeviceToHost)); p += (size_t)B * mb;
  HIP_TRY(hipMemcpy(p, s->d_free, (size_t)n_pages * sizeof(int32_t), hipMemcpyDeviceToHost));
  return MPK_OK;
}

extern "C" const float* mpk_serve_logits(const mpk_server* s) { return s ? s->d_logits : nullptr; }

extern "C" void mpk_serve_destroy(mpk_server* s) {
  if (!s) return;
  (void)hipSetDevice(s->g->device);
  (void)hipDeviceSynchronize();
  const void* none[2] = {nullptr, nullptr};
  for (mpk_graph* x : s->graphs) {
    (void)hipMemcpy((char*)x->d_const + offsetof(GraphConst, page_table), none, sizeof(none), hipMemcpyHostToDevice);
    x->page_table = nullptr;
    x->server = nullptr;
  }
  server_free(s);
  delete s;
}

extern "C" const char* mpk_last_error(void) { return mpk::last_error(); }

extern "C" void mpk_graph_destroy(mpk_graph* g) {
  if (!g) return;
  if (g->server) mpk_serve_destroy(g->server);
  if (!g->host_only) {
    (void)hipSetDevice(g->device);
    (void)hipDeviceSynchronize();
    free_device(g);
  }
  delete g;
}
