// Device side of the runtime (paper Section 5): the task bodies, the event protocol, the scheduler
// wavefronts and the three kernel templates.  Included by variants.hip, which instantiates the
// kernels, and by runtime.hip (host side), which only needs the argument structures.
//
// One persistent kernel: worker workgroups (one per CU, 512 threads = 8 wavefronts) walk their
// pre-enqueued (ahead-of-time) task list; before a task they wait until its dependent event's
// counter has reached epoch * required, after it they publish their stores and add one to the
// triggering event's counter.  Event counters only ever grow (no reset between steps).
//
// Memory ordering (the GPU has 8 XCDs with private, mutually non-coherent L2s).  Whole-cache
// write-back / invalidate fences cost tens of microseconds per hop with 256 workgroups, so the
// runtime never issues them.  Instead every datum that crosses workgroups inside the kernel
// (activations, split-KV partials, the K/V row appended this step, event counters) is written
// with agent-scope stores and read with agent-scope loads (ld_act / st_act below): such accesses
// are performed at the device coherence point, not in an XCD-private cache.  Producer side:
// agent-scope stores, every wavefront waits for its own stores to complete (vmcnt 0), workgroup
// barrier, one lane adds to the event counter.  Consumer side: one lane polls the counter,
// workgroup barrier, then agent-scope loads.  Weights, descriptors and cache rows of earlier
// steps are immutable during a step and use ordinary (non-temporal) loads.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "mpk_internal.h"

namespace mpk {
const char* last_error();
size_t export_size(const HostGraph& g);
void export_graph(const HostGraph& g, void* buf);

// Everything that is fixed for the lifetime of a graph lives in one device-resident record that
// the kernels reach through a pointer (uniform address -> scalar loads on demand, nothing is
// pinned in registers for the whole kernel).
struct GraphConst {
  const TaskDesc* tasks;
  const EventDesc* events;
  uint32_t* counters;
  uint32_t* hier;            // counter blocks of hierarchical events
  const uint32_t* aot_off;
  const uint32_t* aot;
  const uint32_t* op_list;   // per-operator launch: task indices grouped by operator
  uint32_t* err;             // [0] error code, [1] abort flag, [2..3] detail
  const double* inv_freq;    // RoPE frequencies theta^(-2i/d), i < head_dim / 2
  uint32_t* grp_counters;    // arrival counters per (layer, sequence, KV head), monotonic
  uint64_t* trace;           // optional [n_tasks][kTraceSlots] timestamps (100 MHz), or null
  uint64_t timeout_ticks;
  uint32_t n_workers;
  uint32_t vocab, max_seq, n_q, n_kv, head_dim, batch;
  uint32_t lin_rows_max;     // largest number of weight rows (gate/up pairs count twice) of a linear task
  uint32_t lin_res_rows_max; // largest number of columns of a linear task that adds a residual
  uint32_t lin_page_off;     // float offset of the LDS pre-load pages in the task area (0: none)
  // just-in-time launch (Section 5.2): scheduler event queues and worker task queues.  Entries
  // are 64-bit (ticket + 1) << 32 | id with tickets that only grow, so a slot is valid exactly
  // when it carries the ticket its reader expects; tails sit on their own 256-byte lines.
  uint32_t n_sched;          // scheduler wavefronts (0: every task is ahead-of-time)
  uint32_t evq_cap, wq_cap;  // powers of two
  uint64_t* evq_buf;         // [n_sched][evq_cap]
  uint32_t* evq_tail;        // [n_sched][64]
  uint32_t* sched_state;     // [n_sched][64]: [0] head ticket, [1] round-robin cursor (persist across steps)
  const uint32_t* sched_nev; // [n_sched] events a scheduler handles per step
  uint64_t* wq_buf;          // [n_workers][wq_cap]
  uint32_t* wq_tail;         // [n_workers][64]
  uint32_t* wq_head;         // [n_workers] head ticket (persists across steps)
  uint32_t start_event, terminal_event;
  // multi-token launch: written by mpk_decode_steps before the launch (stream-ordered copy)
  int32_t* tokens_out;   // [n_steps][batch] or null
  float* logits_all;     // [n_steps][batch][vocab] or null
  // paged KV cache (Section 6.1): row r of sequence b lives in page page_table[b][r >> page_shift]
  // of the layer's pool [kv_pages][n_kv][1 << page_shift][head_dim]; the table is device memory
  // that the serving task (or the caller, between launches) writes
  const int32_t* page_table;   // [batch][max_seq >> page_shift], or null
  const ServeDev* serve;       // serving state, or null
  uint32_t page_shift, kv_pages;
  int32_t serve_event;         // event the serving task triggers, -1 = none
};

// Per-step kernel arguments, passed by value.  Every device function taking it is force-inlined:
// a real call with a reference to it would make the compiler copy the struct to private memory.
// Tables that no kernel ever writes (the graph record, task and event descriptors, queues) are
// read through the constant address space: uniform reads then become scalar loads, which use
// their own counter and never queue behind (or wait for) the vector-memory weight stream.
#define MPK_CONST __attribute__((address_space(4)))
struct StepArgs {
  const MPK_CONST GraphConst* g;
  // what every wait and notification needs, by value: kernel arguments are in scalar registers
  // when the kernel starts, a field behind `g` costs a memory round trip on the critical path
  const TaskDesc* tasks;
  const EventDesc* events;
  uint32_t* counters;
  uint32_t* hier;
  uint32_t n_sched;
  uint32_t epoch;
  const int32_t* token_ids;
  const int32_t* positions;
  float* logits;
  // multi-token launch (greedy_loop graphs): the kernel runs n_steps decode steps; `step` counts
  // them and `epoch` grows with it.  positions[] stays as the host wrote it until the last step
  // (tasks run ahead of the sampling, so they take positions[b] + step).  16 bits each: the
  // struct is passed by value to every non-inlined task function and its fields sit in scalar
  // registers throughout the kernel; 16 bytes more of it slowed the single-step launch by 1 to 4 %.
  // For the same reason the output pointers of a multi-token launch and the trace buffer are in
  // the graph record instead.
  uint16_t step, n_steps;
  uint32_t flags;   // kTraceBit
};
static_assert(sizeof(StepArgs) == 80, "StepArgs grew: check the single-step launch time");

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A struct passed by value to a real (non-inlined) function travels through private memory and
// arrives in vector registers: to the compiler every field is then a per-lane value, so the
// descriptor reads behind it become vector loads and every branch on them an exec-mask branch.
// All lanes hold the same values: say so, field by field.
__device__ __forceinline__ uint32_t uniform_u32(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename P>
__device__ __forceinline__ P uniform_ptr(P p) {
  const uint64_t v = (uint64_t)p;
  return (P)(((uint64_t)uniform_u32((uint32_t)(v >> 32)) << 32) | uniform_u32((uint32_t)v));
}
__device__ __forceinline__ StepArgs uniform_args(const StepArgs& a) {
  StepArgs u;
  u.g = uniform_ptr(a.g);
  u.tasks = uniform_ptr(a.tasks);
  u.events = uniform_ptr(a.events);
  u.counters = uniform_ptr(a.counters);
  u.hier = uniform_ptr(a.hier);
  u.n_sched = uniform_u32(a.n_sched);
  u.epoch = uniform_u32(a.epoch);
  u.token_ids = uniform_ptr(a.token_ids);
  u.positions = uniform_ptr(a.positions);
  u.logits = uniform_ptr(a.logits);
  u.step = (uint16_t)uniform_u32(a.step);
  u.n_steps = (uint16_t)uniform_u32(a.n_steps);
  u.flags = uniform_u32(a.flags);
  return u;
}

// Pointers that arrive through descriptors in memory are "generic" to the compiler, which then
// emits FLAT memory instructions: those may complete out of order, so every use has to wait for
// ALL outstanding memory operations (vmcnt(0) lgkmcnt(0)) and nothing pipelines.  Everything the
// kernels touch outside LDS is device memory: say so, and loads/stores become GLOBAL instructions
// that complete in order and can be waited for one by one.
#define MPK_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ MPK_GLOBAL T* as_global(T* p) {
  return (MPK_GLOBAL T*)p;
}
// 16-byte non-temporal load (weights, cache rows: streamed once, keep them out of the caches)
__device__ __forceinline__ u32x4 ld_stream16(const void* p) {
  return __builtin_nontemporal_load(as_global((const u32x4*)p));
}

template <typename T>
__device__ __forceinline__ T ld_const_record(const T* p) {   // sizeof(T) a multiple of 16
  union {
    T rec;
    u32x4 v[sizeof(T) / 16];
  } u;
  const MPK_CONST u32x4* src = (const MPK_CONST u32x4*)p;
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 16; ++i) u.v[i] = src[i];
  return u.rec;
}
__device__ __forceinline__ TaskDesc ld_task(const StepArgs& a, uint32_t i) { return ld_const_record(a.tasks + i); }
__device__ __forceinline__ uint32_t ld_u32c(const uint32_t* p) { return *(const MPK_CONST uint32_t*)p; }

constexpr int kTraceSlots = 12;
// StepArgs::flags
constexpr uint32_t kTraceBit = 1u;      // per-task timestamps are recorded (buffer: GraphConst::trace)
constexpr uint32_t kJitterBit = 2u;     // every task starts after a pseudo-random delay (race hunting)
constexpr uint32_t kNoPreloadBit = 4u;  // no weight / cache-row request before a task's event wait
constexpr uint32_t kLoseNotifyBit = 8u; // worker 0 drops its notifications in this launch (watchdog test)
constexpr uint32_t kServeBit = 16u;     // serving launch: positions[] and token_ids[] are rewritten by the serving
                                        // task at the start of every step (absolute positions, read coherently)
constexpr uint32_t kOneStepBit = 32u;   // the launch runs ONE step (single-step entry points, a launch per step of a run):
                                        // nothing that earlier steps wrote can be stale in a cache
__device__ __forceinline__ void trace_mark(const StepArgs& a, const TaskDesc& t, int slot) {
  if ((a.flags & kTraceBit) && threadIdx.x == 0) as_global(a.g->trace)[(size_t)t.pad * kTraceSlots + slot] = wall_clock64();
}

// MPK_DEBUG_JITTER: a delay of 0 .. 20 us, a hash of (task, step), before the task does anything.
// It shifts every task against every other differently in every step, so a consumer that does not
// really wait for its event, or a producer that notifies before its stores have completed, shows
// up as a wrong result instead of depending on the timing of an unloaded machine.
__device__ __forceinline__ void debug_jitter(const StepArgs& a, uint32_t task_index) {
  if (!(a.flags & kJitterBit)) return;
  if (threadIdx.x == 0) {
    uint32_t h = (task_index + 1u) * 2654435761u ^ (a.epoch * 40503u + 0x9E3779B9u);
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    const uint64_t ticks = h % 2000u;   // the wall clock counts at 100 MHz
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(8);
  }
  __syncthreads();
}

enum DevErr : uint32_t { DE_NONE = 0, DE_TIMEOUT = 1, DE_BAD_POSITION = 2, DE_BAD_TOKEN = 3, DE_BAD_META = 4, DE_BAD_PAGE = 5 };

// ------------------------------------------------------------------------------ device helpers
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
// The same sum without LDS traffic: four data-parallel-primitive steps inside each row of 16 lanes
// (lane ^ 1, lane ^ 2, mirror of 8, mirror of 16), then the four row totals.
__device__ __forceinline__ float wave_sum_dpp(float v) {
  auto dpp = [](float x, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  v += dpp(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  v += dpp(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v += dpp(v, std::integral_constant<int, 0x140>{});   // row_mirror
  const int u = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(u, 0)) + __int_as_float(__builtin_amdgcn_readlane(u, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(u, 32)) + __int_as_float(__builtin_amdgcn_readlane(u, 48)));
}
// ... and the largest / smallest value of the wavefront the same way
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce_dpp(uint32_t v, Op op) {
  auto dpp = [](uint32_t x, auto ctrl) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, decltype(ctrl)::value, 0xF, 0xF, true);
  };
  v = op(v, dpp(v, std::integral_constant<int, 0xB1>{}));
  v = op(v, dpp(v, std::integral_constant<int, 0x4E>{}));
  v = op(v, dpp(v, std::integral_constant<int, 0x141>{}));
  v = op(v, dpp(v, std::integral_constant<int, 0x140>{}));
  const int u = (int)v;
  return op(op((uint32_t)__builtin_amdgcn_readlane(u, 0), (uint32_t)__builtin_amdgcn_readlane(u, 16)),
            op((uint32_t)__builtin_amdgcn_readlane(u, 32), (uint32_t)__builtin_amdgcn_readlane(u, 48)));
}
__device__ __forceinline__ float wave_max_dpp(float v) {
  return __uint_as_float(wave_reduce_dpp(__float_as_uint(v), [](uint32_t x, uint32_t y) {
    return __float_as_uint(fmaxf(__uint_as_float(x), __uint_as_float(y)));
  }));
}
__device__ __forceinline__ uint32_t wave_min_u32_dpp(uint32_t v) {
  return wave_reduce_dpp(v, [](uint32_t x, uint32_t y) { return min(x, y); });
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// Sum over the whole workgroup; every thread gets the result.  red: >= 16 floats of LDS.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < (int)(kThreads / 64); ++i) s += red[i];
  return s;
}

// Agent-coherent accessors for data produced and consumed by different workgroups in one launch.
__device__ __forceinline__ float ld_act(const float* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_act(float* p, float v) {
  __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_act2(const float* p) {   // p 8-byte aligned
  uint64_t u = __hip_atomic_load(as_global((const uint64_t*)p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32)));
}
__device__ __forceinline__ uint32_t ld_relaxed(const uint32_t* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_relaxed64(const uint64_t* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_act_u32(uint32_t* p, uint32_t v) {
  __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u32x4 ld_row16_coherent(const uint16_t* p) {   // p 16-byte aligned
  uint64_t a = __hip_atomic_load(as_global((const uint64_t*)p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  uint64_t b = __hip_atomic_load(as_global((const uint64_t*)p + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return u32x4{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
}

__device__ __forceinline__ float dot8(const u32x4& w, const float4& x0, const float4& x1, float acc) {
  acc = fmaf(bf16_lo(w.x), x0.x, acc);
  acc = fmaf(bf16_hi(w.x), x0.y, acc);
  acc = fmaf(bf16_lo(w.y), x0.z, acc);
  acc = fmaf(bf16_hi(w.y), x0.w, acc);
  acc = fmaf(bf16_lo(w.z), x1.x, acc);
  acc = fmaf(bf16_hi(w.z), x1.y, acc);
  acc = fmaf(bf16_lo(w.w), x1.z, acc);
  acc = fmaf(bf16_hi(w.w), x1.w, acc);
  return acc;
}

__device__ __forceinline__ void report(const StepArgs& a, uint32_t code, uint32_t d0, uint32_t d1) {
  if (atomicCAS(&a.g->err[0], 0u, code) == 0u) {
    a.g->err[2] = d0;
    a.g->err[3] = d1;
  }
}

// ------------------------------------------------------------------------------ task bodies
// T0: x[b] = E[token[b]] widened to fp32.
__device__ __forceinline__ void body_embed(const TaskDesc& t, const StepArgs& a) {
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    int32_t tok = (int32_t)ld_relaxed((const uint32_t*)a.token_ids + b);   // may come from the previous step's sampling task
    if (tok < 0 || (uint32_t)tok >= a.g->vocab) {
      if (threadIdx.x == 0) report(a, DE_BAD_TOKEN, b, (uint32_t)tok);
      tok = 0;
    }
    const uint16_t* row = (const uint16_t*)t.w + (size_t)tok * t.K;
    float* out = t.out + (size_t)b * t.ld_out;
    for (uint32_t i = threadIdx.x; i < t.K; i += kThreads) st_act(out + i, bf16_to_f32(as_global(row)[i]));
  }
}

// T1/T8/T13: y = x * (1 / sqrt(mean(x^2) + eps)) * g, one batch row per task.
__device__ __forceinline__ void body_rmsnorm(const TaskDesc& t, float* lds) {
  const uint16_t* g = (const uint16_t*)t.w2;
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    const float* x = t.in + (size_t)b * t.ld_in;
    float* y = t.out + (size_t)b * t.ld_out;
    float ss = 0.f;
    for (uint32_t i = threadIdx.x; i < t.K; i += kThreads) {
      float v = ld_act(x + i);
      ss = fmaf(v, v, ss);
    }
    ss = block_sum(ss, lds);
    float inv = 1.0f / sqrtf(ss / (float)t.K + t.f0);
    for (uint32_t i = threadIdx.x; i < t.K; i += kThreads) st_act(y + i, ld_act(x + i) * inv * bf16_to_f32(as_global(g)[i]));
  }
}

__device__ __forceinline__ bool wait_event(const StepArgs& a, int32_t e, uint32_t* s_flag);

// ------------------------------------------------------------------------------ linear tasks
// T2/T6/T9/T11/T14: y[b][c] = sum_j W[c][j] x[b][j] for output columns [c0, c1), all batch rows
// at once, with optional fused stages: RMSNorm of the input (TF_PRO_NORM), residual add
// (TF_EPI_RESID), silu(gate) * up (TF_GATEUP: column c needs weight rows c and F + c).
//
// Weight rows of a task ("ring rows": one per column, or the (gate, up) pair of each column) are
// split into 8 contiguous ranges, one per wavefront.  A wavefront walks its rows in pairs and
// every pair in segments of 4096 input elements; one (pair, segment) is a half block of
// 2 rows x 8 stages, a stage being 64 lanes x 16 bytes = 512 elements: 16 sixteen-byte loads per
// lane.  A wavefront owns two half-block buffers (32 KB, 256 KB per CU) and uses them in turn: it
// consumes one, requests that buffer's next half block at once, and turns to the other.  The
// compiler's count of the loads in flight does not survive the loop's back edge (it waits for
// both buffers before the first use of either), so a wavefront still drains its queue once per
// pair of half blocks; the eight wavefronts of a CU drift apart and cover for each other.
// Against ONE buffer of twice the size, requested whole and then consumed whole: the first
// buffer's request goes out half a block earlier, and a task with two rows per wavefront (the O
// and down projections of the 8B shape) pre-loads two segments instead of one.
//
// Cross-task pipelining (paper Section 5.3).  Weights never depend on an event, so a task
// requests its first two half blocks (256 KB per CU) BEFORE it waits for its dependent event:
// they stream in while the input vector is still being produced elsewhere.  At the end of a task
// wavefront 0 alone applies the epilogue, writes the outputs with coherent stores and waits for
// exactly those stores; the other wavefronts wait at a barrier meanwhile, and only then walk into
// the worker's next task and issue its first requests, while wavefront 0 notifies the triggering
// event, requests its own share and polls the next event.  (The others must not run ahead: all
// wavefronts of a CU share its path to memory, and output stores queued behind their requests
// were acknowledged up to 10 us late.)
// The buffers are local to a task on purpose: carried around the task loop instead, the
// compiler moves parts of them to scratch memory, and a scratch access in the middle of a request
// waits for every load issued before it.
constexpr int kHalfRows = 2, kRingStages = 8;
constexpr uint32_t kSegLen = 512u * kRingStages;   // input elements per half-block row
struct HalfRing {
  u32x4 s[kHalfRows][kRingStages];
};

__device__ __forceinline__ void ring_clear(HalfRing& ring) {
#pragma unroll
  for (int i = 0; i < kHalfRows; ++i)
#pragma unroll
    for (int u = 0; u < kRingStages; ++u) ring.s[i][u] = u32x4{0, 0, 0, 0};
}

// Wavefront-uniform view of one linear task for one wavefront.
struct LinGeom {
  const uint16_t* W;
  uint32_t K, c0, F, gateup;
  uint32_t r0, r1;    // ring rows [r0, r1) of this wavefront within the task
  uint32_t nseg;      // segments per row
};

__device__ __forceinline__ LinGeom lin_geom(const TaskDesc& t, uint32_t wave) {
  LinGeom g;
  g.W = (const uint16_t*)t.w;
  g.K = t.K;
  g.c0 = t.c0;
  g.F = t.p0;
  g.gateup = (t.flags & TF_GATEUP) ? 1u : 0u;
  const uint32_t R = (t.c1 - t.c0) << g.gateup;
  constexpr uint32_t NW = kThreads / 64;
  // rows are dealt in pairs (a half block holds two; a (gate, up) pair stays in one wavefront):
  // every wavefront gets floor(pairs / 8) of them and the first pairs % 8 wavefronts one more, so
  // that a tile of any size -- tiles sized by worker speed are seldom multiples of 16 rows --
  // loads the wavefronts to within one pair of each other
  const uint32_t P = (R + 1u) / 2u, base = P / NW, extra = P % NW;
  const uint32_t p0 = wave * base + min(wave, extra), p1 = p0 + base + (wave < extra ? 1u : 0u);
  g.r0 = min(2u * p0, R);
  g.r1 = min(2u * p1, R);
  g.nseg = (t.K + kSegLen - 1u) / kSegLen;
  return g;
}

// Position of a wavefront in its sequence of half blocks: rows [row0, row0 + 2) x segment `seg`,
// segments of a pair first.  Two of them walk the sequence: one requests, one consumes.
struct LinCursor {
  uint32_t row0, seg;
};
__device__ __forceinline__ bool lin_valid(const LinGeom& g, const LinCursor& c) { return c.row0 < g.r1; }
__device__ __forceinline__ void lin_advance(const LinGeom& g, LinCursor& c) {
  if (++c.seg == g.nseg) {
    c.seg = 0;
    c.row0 += kHalfRows;
  }
}

// The half block at a cursor.
struct LinHalf {
  const uint16_t* p[kHalfRows];   // row start + segment start (a second row past the end repeats the first)
  uint32_t row0, nrows, seg, seglen;
};

__device__ __forceinline__ LinHalf lin_half(const LinGeom& g, const LinCursor& c) {
  LinHalf B;
  B.seg = c.seg;
  B.row0 = c.row0;
  B.nrows = min(g.r1 - c.row0, (uint32_t)kHalfRows);
  B.seglen = min(kSegLen, g.K - c.seg * kSegLen);
#pragma unroll
  for (int i = 0; i < kHalfRows; ++i) {
    const uint32_t r = B.row0 + min((uint32_t)i, B.nrows - 1u);
    const uint32_t wrow = g.gateup ? (g.c0 + (r >> 1) + ((r & 1u) ? g.F : 0u)) : g.c0 + r;
    B.p[i] = g.W + (size_t)wrow * g.K + c.seg * kSegLen;
  }
  return B;
}

// Requests a half block, stage by stage.  Lanes past the end of a short segment re-read its last
// 16 bytes (the staged input is zero there), so every lane takes part in every load.
__device__ __forceinline__ void lin_request(const LinHalf& B, HalfRing& ring, int lane) {
  if (B.seglen == kSegLen) {   // full segment: one base address per row, constant stage offsets
#pragma unroll
    for (int u = 0; u < kRingStages; ++u)
#pragma unroll
      for (int i = 0; i < kHalfRows; ++i) ring.s[i][u] = ld_stream16(B.p[i] + lane * 8 + u * 512);
  } else {
#pragma unroll
    for (int u = 0; u < kRingStages; ++u) {
      const uint32_t o = min((uint32_t)u * 512u + (uint32_t)lane * 8u, B.seglen - 8u);
#pragma unroll
      for (int i = 0; i < kHalfRows; ++i) ring.s[i][u] = ld_stream16(B.p[i] + o);
    }
  }
}

// Adds the half block's partial dot products to acc.
template <int NB>
__device__ __forceinline__ void lin_consume(const LinHalf& B, const HalfRing& ring, const float* xs, uint32_t Kp,
                                            int lane, float (&acc)[kHalfRows][NB]) {
#pragma unroll
  for (int u = 0; u < kRingStages; ++u) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const float4* xp = (const float4*)(xs + (size_t)b * Kp + B.seg * kSegLen + u * 512 + lane * 8);
      const float4 x0 = xp[0], x1 = xp[1];
#pragma unroll
      for (int i = 0; i < kHalfRows; ++i) acc[i][b] = dot8(ring.s[i][u], x0, x1, acc[i][b]);
    }
  }
}

// LDS pre-load pages (paper Section 5.3: data of a task that has not started yet is pre-loaded into
// shared-memory pages).  One page per wavefront holds one half block in the layout of a HalfRing:
// [row 0..1][stage 0..7][lane] x 16 bytes.  The loads go from device memory straight into LDS (no
// registers), so a page can be filled by one task and consumed by the worker's next one.
typedef __attribute__((address_space(3))) void* lds_ptr_t;
__device__ __forceinline__ void lin_request_page(const LinHalf& B, u32x4* page, int lane) {
#pragma unroll
  for (int u = 0; u < kRingStages; ++u) {
    const uint32_t o = min((uint32_t)u * 512u + (uint32_t)lane * 8u, B.seglen - 8u);
#pragma unroll
    for (int i = 0; i < kHalfRows; ++i)
      __builtin_amdgcn_global_load_lds(as_global((const u32x4*)(B.p[i] + o)), (lds_ptr_t)(page + (i * kRingStages + u) * 64), 16, 0, 0);
  }
}
template <int NB>
__device__ __forceinline__ void lin_consume_page(const LinHalf& B, const u32x4* page, const float* xs, uint32_t Kp,
                                                 int lane, float (&acc)[kHalfRows][NB]) {
#pragma unroll
  for (int u = 0; u < kRingStages; ++u) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const float4* xp = (const float4*)(xs + (size_t)b * Kp + B.seg * kSegLen + u * 512 + lane * 8);
      const float4 x0 = xp[0], x1 = xp[1];
#pragma unroll
      for (int i = 0; i < kHalfRows; ++i) acc[i][b] = dot8(page[(i * kRingStages + u) * 64 + lane], x0, x1, acc[i][b]);
    }
  }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() carries a release fence, for
// which the compiler drains the vector-memory queue (s_waitcnt vmcnt(0)): with a pre-load of
// the next task in flight that would stall every wavefront, and the event notification behind
// it, until the whole pre-load has landed.  What the barriers of a linear task publish lives in
// LDS; data for other workgroups is published by wavefront 0 with its own wait.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ void signal_from_wave0(const StepArgs& a, const TaskDesc& t, int32_t e, int lane);
__device__ __forceinline__ void notify_event(const StepArgs& a, int32_t e);
__device__ __forceinline__ void poll_event_wave0(const StepArgs& a, int32_t e, uint32_t* s_flag, int lane);
__device__ __forceinline__ void poll_event_or_jit_wave0(const StepArgs& a, int32_t e, uint32_t* s_flag, int lane, uint32_t jit_head);
// Hybrid launch (Section 5.2): a worker may start the linear task at the head of its ahead-of-time
// queue before that task's event is activated (so the weights are requested early), provided it
// keeps an eye on its just-in-time queue while it waits: a worker that blocked regardless could
// sit on the very tasks the awaited event depends on.  When a just-in-time task arrives first,
// the linear task gives up (kLinPreempted, task index in s_flag[1]); the worker runs that task and
// starts the linear task again.  (Running it from inside the wait would keep the pre-loaded
// weights live across a call: the compiler then moves them to scratch memory for good.)
// NoJit: all-ahead-of-time kernels, nothing to watch.
constexpr uint32_t kLinAbort = 0, kLinDone = 1, kLinPreempted = 2;
struct NoJit {
  static constexpr bool enabled = false;
  uint32_t jit_head = 0;
};
struct JitWatch {
  static constexpr bool enabled = true;
  uint32_t jit_head;   // the worker's consumer ticket of its just-in-time queue
};
// The wait of a linear task for its dependent event: kLinDone (activated), kLinAbort, kLinPreempted.
template <class Svc>
__device__ __forceinline__ uint32_t linear_wait(const StepArgs& a, int32_t wait_ev, uint32_t* s_flag, uint32_t wave, int lane,
                                                const Svc& svc) {
  if (wave == 0) {
    if constexpr (Svc::enabled) poll_event_or_jit_wave0(a, wait_ev, s_flag, lane, svc.jit_head);
    else poll_event_wave0(a, wait_ev, s_flag, lane);
  }
  lds_barrier();
  return __builtin_amdgcn_readfirstlane(*s_flag);   // (uniform; tell the compiler)
}

// LDS layout of a linear task (floats): xs [NB][K rounded up to 4096] | outbuf [max ring rows][NB]
// | resid [max columns][NB] | ssq [8][NB]; the two middle regions are sized by the compiler from
// the largest task of the graph (GraphConst::lin_rows_max).
//
// Runs task `t`.  wait_ev >= 0: wait for that event first (persistent kernel).  Returns whether
// the step is still alive (false: watchdog / abort).
template <int NB, bool MEGA, class Svc = NoJit, bool DEEP = false>
__device__ __forceinline__ uint32_t linear_task(const TaskDesc& t, const StepArgs& a, float* lds, int32_t wait_ev,
                                                uint32_t* s_flag, const Svc& svc = Svc{}, uint32_t next_ti = 0) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: geometry stays scalar
  const uint32_t K = t.K, nb = t.b1 - t.b0, ncols = t.c1 - t.c0;
  // pages exist only in the all-ahead-of-time persistent kernel at batch 1 (the compiler sets the flags)
  constexpr bool kPages = MEGA && NB == 1 && !Svc::enabled;
  u32x4* page = (u32x4*)(lds + a.g->lin_page_off) + (size_t)wave * (kLinPageFloats / 4);
  const bool page_ready = kPages && (t.flags & TF_PAGE_READY), page_next = kPages && (t.flags & TF_PAGE_NEXT);
  const uint32_t Kp = (K + kSegLen - 1u) / kSegLen * kSegLen;
  const uint32_t rows_max = a.g->lin_rows_max;
  float* xs = lds;                                   // [NB][Kp]
  float* outbuf = xs + (size_t)NB * Kp;              // [rows_max][NB]
  float* res_lds = outbuf + (size_t)rows_max * NB;   // [rows_max][NB]
  float* ssq = res_lds + (size_t)rows_max * NB;      // [8][NB]
  const LinGeom g = lin_geom(t, wave);
  HalfRing h0, h1;   // local to the task: nothing is live around the task loop, so they stay in registers
  ring_clear(h0);
  ring_clear(h1);
  LinCursor rq{g.r0, 0u};   // next half block to request
  if (page_ready && lin_valid(g, rq)) lin_advance(g, rq);   // the first one is in this wavefront's page already
  // (every request site ends in an (empty) assembly statement of its own: otherwise the compiler
  // may merge the identical last loads of two sites into one whose destination is chosen at run
  // time, and a buffer addressed that way is moved from registers to scratch memory)
  const bool preload = !(a.flags & kNoPreloadBit);   // off: the ablation of Section 6.5, Fig. 10
  if (preload && lin_valid(g, rq)) {
    lin_request(lin_half(g, rq), h0, lane);
    lin_advance(g, rq);
    asm volatile("; first half block requested" ::: "memory");
  }
  if (preload && lin_valid(g, rq)) {
    lin_request(lin_half(g, rq), h1, lane);
    lin_advance(g, rq);
    asm volatile("; second half block requested" ::: "memory");
  }
  // DEEP: a third buffer -- 384 KB per CU requested before the event and a deeper queue while
  // streaming.  A kernel variant of its own, picked for models whose linear tasks are large (70B
  // shape: -3 % per step); small tasks are bound by the hops between operators, where a bigger
  // burst ahead of the event poll and the input loads only delays those (8B shape: +3 %), and the
  // mere presence of the third buffer in the kernel costs the small shape 2 %.
  constexpr bool kThird = DEEP;
  HalfRing h2;
  if (kThird) {
    ring_clear(h2);
    if (preload && lin_valid(g, rq)) {
      lin_request(lin_half(g, rq), h2, lane);
      lin_advance(g, rq);
      asm volatile("; third half block requested" ::: "memory");
    }
  }
  // the first gains of a folded RMSNorm are weights too: requested before the event, so that the
  // staging below is one round trip (the input) instead of two
  constexpr int kGainPre = 4;   // x 512 threads x 2: the first 4096 inputs
  uint32_t gpre[kGainPre];
  {
    const uint16_t* gain0 = (const uint16_t*)t.w2;
#pragma unroll
    for (int u = 0; u < kGainPre; ++u) {
      const uint32_t i = u * kThreads + threadIdx.x;
      gpre[u] = 0;
      if ((t.flags & TF_PRO_NORM) && i < K / 2) gpre[u] = *as_global((const uint32_t*)(gain0 + 2 * i));
    }
  }
  if (page_next) {
    // this task is short and has a long wait ahead: the first half block of every wavefront's
    // share of the worker's NEXT task goes into the pages now, two tasks ahead of its use
    const TaskDesc tn = ld_task(a, next_ti);
    const LinGeom gn = lin_geom(tn, wave);
    const LinCursor cn{gn.r0, 0u};
    if (lin_valid(gn, cn)) lin_request_page(lin_half(gn, cn), page, lane);
  }
  // ---- dependent event: wavefront 0 polls, the others wait at the barrier
  if (wait_ev >= 0) {
    const uint32_t w = linear_wait(a, wait_ev, s_flag, wave, lane, svc);
    if (w != kLinDone) return w;   // aborted, or pre-empted by a just-in-time task: the requested weights are dropped
  }
  trace_mark(a, t, 1);
  if (!preload) {   // pre-loading switched off: the first requests go out only now
    if (lin_valid(g, rq)) {
      lin_request(lin_half(g, rq), h0, lane);
      lin_advance(g, rq);
      asm volatile("; first half block requested after the event" ::: "memory");
    }
    if (lin_valid(g, rq)) {
      lin_request(lin_half(g, rq), h1, lane);
      lin_advance(g, rq);
      asm volatile("; second half block requested after the event" ::: "memory");
    }
    if (kThird && lin_valid(g, rq)) {
      lin_request(lin_half(g, rq), h2, lane);
      lin_advance(g, rq);
      asm volatile("; third half block requested after the event" ::: "memory");
    }
  }
  // ---- stage the input rows in LDS.  With TF_PRO_NORM the gain is folded in here (x * g) and
  // the row's 1/rms factor is applied to the finished dot products: W (x g inv) = inv * W (x g).
  const bool pro_norm = t.flags & TF_PRO_NORM;
  const uint16_t* gain = (const uint16_t*)t.w2;
  // the residual slice of this tile goes out first (tile-local, small): its round trip then
  // overlaps the staging instead of following it
  const bool resid = t.flags & TF_EPI_RESID;
  float resv = 0.f;
  if (resid && threadIdx.x < nb * ncols) {
    const uint32_t bb = threadIdx.x / ncols, cc = threadIdx.x % ncols;
    resv = ld_act(t.in2 + (size_t)(t.b0 + bb) * t.ld_out + t.c0 + cc);
  }
  constexpr int kStageLoads = 12;   // coherent loads in flight per lane: 12288 inputs in one round trip
#pragma unroll
  for (uint32_t b = 0; b < (uint32_t)NB; ++b) {
    float2* dst = (float2*)(xs + (size_t)b * Kp);
    float ss = 0.f;
    if (b < nb) {
      const float* src = t.in + (size_t)(t.b0 + b) * t.ld_in;
      for (uint32_t i0 = 0; i0 < Kp / 2; i0 += kThreads * kStageLoads) {
        float2 tmp[kStageLoads];
#pragma unroll
        for (int u = 0; u < kStageLoads; ++u) {
          uint32_t i = i0 + u * kThreads + threadIdx.x;
          if (i < K / 2) tmp[u] = ld_act2(src + 2 * i);
        }
#pragma unroll
        for (int u = 0; u < kStageLoads; ++u) {
          uint32_t i = i0 + u * kThreads + threadIdx.x;
          if (i < K / 2) {
            float2 v = tmp[u];
            if (pro_norm) {
              ss = fmaf(v.x, v.x, ss);
              ss = fmaf(v.y, v.y, ss);
              uint32_t g2 = (i0 == 0 && u < kGainPre) ? gpre[u < kGainPre ? u : 0] : *as_global((const uint32_t*)(gain + 2 * i));
              v.x *= bf16_lo(g2);
              v.y *= bf16_hi(g2);
            }
            dst[i] = v;
          } else if (i < Kp / 2) {
            dst[i] = make_float2(0.f, 0.f);
          }
        }
      }
    } else {
      for (uint32_t i = threadIdx.x; i < Kp / 2; i += kThreads) dst[i] = make_float2(0.f, 0.f);
    }
    if (pro_norm) {
      ss = wave_sum_dpp(ss);
      if (lane == 0) ssq[wave * NB + b] = ss;
    }
  }
  if (resid) {
    if (threadIdx.x < nb * ncols) res_lds[threadIdx.x] = resv;
    for (uint32_t i = threadIdx.x + kThreads; i < nb * ncols; i += kThreads) {   // more than 512 outputs per task: rare
      uint32_t bb = i / ncols, cc = i % ncols;
      res_lds[i] = ld_act(t.in2 + (size_t)(t.b0 + bb) * t.ld_out + t.c0 + cc);
    }
  }
  lds_barrier();
  trace_mark(a, t, 2);
  // ---- stream this wavefront's rows: the two buffers in turn
  {
    float acc[kHalfRows][NB];
#pragma unroll
    for (int i = 0; i < kHalfRows; ++i)
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[i][b] = 0.f;
    // the pair of rows is complete with its last segment: reduce across lanes, results to LDS
    auto finish = [&](const LinHalf& B) {
      if (B.seg + 1 == g.nseg) {
#pragma unroll
        for (int i = 0; i < kHalfRows; ++i)
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const float v = wave_sum_dpp(acc[i][b]);
            if (lane == 0 && (uint32_t)i < B.nrows) outbuf[(size_t)(B.row0 + i) * NB + b] = v;
            acc[i][b] = 0.f;
          }
      }
    };
    LinCursor cs{g.r0, 0u};
    if (page_ready && lin_valid(g, cs)) {   // (requested a whole task ago: long since landed)
      const LinHalf B = lin_half(g, cs);
      lin_consume_page<NB>(B, page, xs, Kp, lane, acc);
      finish(B);
      lin_advance(g, cs);
    }
    while (lin_valid(g, cs)) {
      {
        const LinHalf B = lin_half(g, cs);
        lin_consume<NB>(B, h0, xs, Kp, lane, acc);
        finish(B);
        lin_advance(g, cs);
      }
      if (lin_valid(g, rq)) {
        lin_request(lin_half(g, rq), h0, lane);
        lin_advance(g, rq);
        asm volatile("; first buffer requested again" ::: "memory");
      }
      if (!lin_valid(g, cs)) break;
      {
        const LinHalf B = lin_half(g, cs);
        lin_consume<NB>(B, h1, xs, Kp, lane, acc);
        finish(B);
        lin_advance(g, cs);
      }
      if (lin_valid(g, rq)) {
        lin_request(lin_half(g, rq), h1, lane);
        lin_advance(g, rq);
        asm volatile("; second buffer requested again" ::: "memory");
      }
      if (kThird) {
        if (!lin_valid(g, cs)) break;
        {
          const LinHalf B = lin_half(g, cs);
          lin_consume<NB>(B, h2, xs, Kp, lane, acc);
          finish(B);
          lin_advance(g, cs);
        }
        if (lin_valid(g, rq)) {
          lin_request(lin_half(g, rq), h2, lane);
          lin_advance(g, rq);
          asm volatile("; third buffer requested again" ::: "memory");
        }
      }
    }
  }
  lds_barrier();
  trace_mark(a, t, 3);
  // ---- wavefront 0: epilogue, outputs, notification, then its own share of the pre-load
  if (wave == 0) {
    float* outp = (t.flags & TF_OUT_LOGITS) ? a.logits : t.out;
    float inv_rms[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      inv_rms[b] = 1.0f;
      if (pro_norm && (uint32_t)b < nb) {
        float ss = 0.f;
#pragma unroll
        for (int w = 0; w < (int)(kThreads / 64); ++w) ss += ssq[w * NB + b];
        inv_rms[b] = 1.0f / sqrtf(ss / (float)K + t.f0);
      }
    }
    for (uint32_t i = lane; i < ncols * nb; i += 64) {
      const uint32_t cc = i % ncols, bb = i / ncols;
      float inv = inv_rms[0];
#pragma unroll
      for (int b = 1; b < NB; ++b) inv = (bb == (uint32_t)b) ? inv_rms[b] : inv;
      float v;
      if (g.gateup) {
        const float gte = outbuf[(size_t)(2 * cc) * NB + bb] * inv, up = outbuf[(size_t)(2 * cc + 1) * NB + bb] * inv;
        v = gte / (1.0f + expf(-gte)) * up;
      } else {
        v = outbuf[(size_t)cc * NB + bb] * inv;
      }
      if (t.flags & TF_EPI_RESID) v = res_lds[bb * ncols + cc] + v;
      st_act(outp + (size_t)(t.b0 + bb) * t.ld_out + t.c0 + cc, v);
    }
    if (MEGA) {   // wait for exactly these stores
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      trace_mark(a, t, 7);
    }
  }
  if (MEGA) {
    // Wavefronts 1..7 issue the next task's requests only now.  Ordering inside ONE wavefront is
    // not enough: all wavefronts of a CU share its path to memory, and behind 224 freshly issued
    // 1 KB loads the few output stores of wavefront 0 were acknowledged up to 10 us late (in-kernel
    // trace), which delays the event for every consumer -- the hop is the critical path, the
    // pre-load has slack.  (Releasing them once the stores have been issued, not acknowledged, was
    // measured too: 0.6 % slower per step on the 8B shape.)
    lds_barrier();
    if (wave == 0) {
      if (t.trig_event >= 0 && lane == 0) notify_event(a, t.trig_event);
      trace_mark(a, t, 4);
    }
  }
  return kLinDone;
}

// ------------------------------------------------------------------------------ linear tasks, batch 5..16
// The same operator for 5 to 16 batch rows, on the matrix cores.  At batch 8 the vector ALUs
// would need about as many cycles for the multiply-adds as HBM needs to deliver the weights; one
// v_mfma_f32_16x16x32_bf16 does 16 weight rows x 32 inputs x 16 batch columns at once.
//   A operand = weights: lane l holds row (l % 16) of a 16-row tile and 8 of the 32 inputs of the
//     multiply: 16 bytes straight from HBM, no conversion (loaded as 8 rows x 128 bytes per
//     instruction and put in place by one DPP move per register: see mfma_job_packed).
//   B operand = activations: lane l holds batch column (l % 16), the same 8 inputs, as bf16.
//     Activations are fp32: x is split into THREE bf16 terms, hi = bf16(x), mid = bf16(x - hi),
//     lo = bf16(x - hi - mid).  Each conversion rounds to nearest and each remainder is exact in
//     fp32, so hi + mid + lo = x exactly (8 + 8 + 8 significand bits), every product with a bf16
//     weight is exact, and the only rounding is the fp32 accumulation -- as in the vector body.
//     (Two terms leave x to 2^-18: logits near zero then miss the element-wise bound.)
//   D: lane l holds batch column (l % 16), tile rows 4 (l / 16) .. + 3.
// The input is staged in LDS as fp32, whole when it fits (4096 inputs up to batch 8, 2048 above;
// longer inputs in chunks of that size), row stride padded by 128 bytes so that the lanes of a
// fragment spread evenly over the banks; the wavefronts split it into the three terms as they go,
// so no barrier separates the staging of one part from the multiplies of another.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t pack_bf16_rne(float x, float y) {   // the hardware's packed conversion
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){x, y}, bf16x2));
}
// (x, y) -> packed bf16 pairs hi, mid, lo with hi + mid + lo = (x, y) exactly
__device__ __forceinline__ void split_hi_mid_lo(float x, float y, uint32_t* hi, uint32_t* mid, uint32_t* lo) {
  const uint32_t h = pack_bf16_rne(x, y);
  const float rx = x - bf16_lo(h), ry = y - bf16_hi(h);
  const uint32_t m = pack_bf16_rne(rx, ry);
  *hi = h;
  *mid = m;
  *lo = pack_bf16_rne(rx - bf16_lo(m), ry - bf16_hi(m));
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Geometry of one matrix-core job: K inputs x nb staged rows x nrt 16-row weight tiles (nrt <= 32).
// Uniform over the wavefront (wave comes from readfirstlane).
//
// The input stays in LDS as fp32, a chunk of up to mfma_kchunk(nb) inputs at a time (the whole of
// it for every operator of the benchmark shapes), so that there is one staging pass and no
// barrier inside the multiply loop; each wavefront turns the 8 inputs x 1 row a lane needs for a
// multiply into the three bf16 terms on the fly.
//
// The 8 wavefronts form rg row groups x ks K slices (rg = 1, 2, 4 or 8, the smallest with
// 4 rg >= nrt).  Wavefront (slice s, group g) owns row tiles g, g + rg, g + 2 rg, g + 3 rg (those
// below nrt: nrtw of them) and, in every chunk, the s-th of ks nearly equal runs of 64-input
// "k-groups".  It works in rounds of 8 weight fragments (32 inputs x 16 rows, 1 KB each) = 4 slot
// groups of kMfmaFrags = 2 fragments, two rounds in flight (16 KB per wavefront, 32 MB over the
// chip: rounds of twice the size keep 64 MB in flight, which HBM does not need and which stands in
// the way of every store acknowledgement, counter update and poll of the hops between operators
// -- 8B shape at batch 8: 5.27 -> 5.10 ms per step; rounds of half the size starve: 5.93);
// slot group q always adds into accumulator q:
//   nrtw >= 3: one k-group per round, slot group q = row tile q of the wavefront
//   nrtw == 2: two k-groups per round, slot group q = (k-group q / 2, row tile q % 2)
//   nrtw == 1: four k-groups per round, slot group q = k-group q
// so the fragments of a k-group's inputs are converted once and used by all row tiles of the
// round.  The epilogue adds the accumulators of a row tile over slot groups and slices in a
// fixed order (mfma_dot).
constexpr uint32_t kMfmaFrags = 2;
struct MfmaGeom {
  uint32_t K, nb, nrt;
  uint32_t Kc, nchunk;   // inputs per chunk, chunks
  uint32_t xstride;      // floats between staged rows
  uint32_t rg, ks;       // row groups x K slices = 8
  uint32_t my_g, my_s;
  uint32_t nrtw;         // row tiles of this wavefront: 0 .. 4
  uint32_t kgpr;         // k-groups per round: 1, 2 or 4
};
__device__ __forceinline__ uint32_t mfma_group_tiles(uint32_t nrt, uint32_t rg, uint32_t g) {
  return g < nrt ? min(4u, (nrt - g + rg - 1u) / rg) : 0u;
}
__device__ __forceinline__ MfmaGeom mfma_geom(uint32_t K, uint32_t nb, uint32_t nrt, uint32_t wave) {
  MfmaGeom G;
  G.K = K; G.nb = nb; G.nrt = nrt;
  G.Kc = mfma_kchunk(nb);
  G.nchunk = (K + G.Kc - 1u) / G.Kc;
  G.xstride = G.Kc + kMfmaXPad;
  uint32_t rg = 1;
  while (4u * rg < nrt && rg < 8u) rg <<= 1;
  G.rg = rg;
  G.ks = 8u / rg;
  G.my_g = wave % rg;
  G.my_s = wave / rg;
  G.nrtw = mfma_group_tiles(nrt, rg, G.my_g);
  G.kgpr = G.nrtw >= 3u ? 1u : (G.nrtw == 2u ? 2u : 4u);
  return G;
}

// 8 consecutive fp32 inputs of one staged row -> packed bf16 terms hi, mid, lo (4 words each)
__device__ __forceinline__ void split8(const float4& p, const float4& q, u32x4* hi, u32x4* mid, u32x4* lo) {
  uint32_t h[4], m[4], l[4];
  split_hi_mid_lo(p.x, p.y, &h[0], &m[0], &l[0]);
  split_hi_mid_lo(p.z, p.w, &h[1], &m[1], &l[1]);
  split_hi_mid_lo(q.x, q.y, &h[2], &m[2], &l[2]);
  split_hi_mid_lo(q.z, q.w, &h[3], &m[3], &l[3]);
  *hi = u32x4{h[0], h[1], h[2], h[3]};
  *mid = u32x4{m[0], m[1], m[2], m[3]};
  *lo = u32x4{l[0], l[1], l[2], l[3]};
}
__device__ __forceinline__ u32x4 select4(bool c, const u32x4& x, const u32x4& y) {
  return u32x4{c ? x.x : y.x, c ? x.y : y.y, c ? x.z : y.z, c ? x.w : y.w};
}

// One job: out[r][b] partial tiles = W rows x staged input rows, left in LDS.
//   wbase, row_off(rt) : weight rows start at wbase (uniform) + row_off(rt) bytes, row_off = this
//                  lane's row of 16-row tile rt (32 bits: a scalar base and one vector offset per
//                  load, no address pairs to keep); loads are clamped to the end of the row
//   src_row(b)   : fp32 input row b (read with coherent loads), b < nb
//   wait_fn()    : called after the first two rounds of weights have been requested (cross-task
//                  pre-loading, Section 5.3: 16 KB per wavefront, 32 MB over the chip); returns
//                  kLinDone to go on
// LDS: x [nb][xstride] f32 at `lds`, reused at the end for the per-wavefront partial tiles
// part[8][4][16][16] f32, then the chunk's RMSNorm gains [Kc] bf16; ssq [8][16] f32 (sums of squares per wavefront and row, when pro_norm).
// On return (kLinDone) every thread may read part and ssq.
// PACK: how many of the three terms one multiply covers.  The multiply has 16 batch columns; up
// to 8 staged rows leave half of them free, so columns 0..7 take the hi term and columns 8..15
// the mid term of the same rows (PACK 2: two multiplies per fragment, the lo term alone in the
// second, on accumulators of its own); up to 4 staged rows take hi | mid | lo in columns 0..3 |
// 4..7 | 8..11 (PACK 3: one multiply).  The column groups are added up once, at the end.
template <int PACK, class RowOff, class SrcRow, class Wait>
__device__ __forceinline__ uint32_t mfma_job_packed(const StepArgs& a, const TaskDesc& t, float* lds, float* ssq, const MfmaGeom& G,
                                                    const uint16_t* wbase, RowOff row_off, SrcRow src_row, bool pro_norm,
                                                    const uint16_t* gain, Wait wait_fn) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t K = G.K, nb = G.nb, nrt = G.nrt, Kc = G.Kc, nchunk = G.nchunk, xstride = G.xstride;
  const uint32_t nrtw = G.nrtw, kgpr = G.kgpr, S = G.ks;
  float* xs = lds;
  float* part = lds;
  const uint32_t frow = lane & 15u, fk = (uint32_t)(lane >> 4) * 8u;
  constexpr uint32_t FR = kMfmaFrags, KG = 32u * FR;   // fragments per slot group, inputs per k-group
  // slot group q of a round: k-group offset inside the round, byte offset of its row tile's row
  const uint32_t sh = kgpr == 4u ? 0u : (kgpr == 2u ? 1u : 2u);   // q >> sh = k-group offset
  // How the weights are loaded.  A multiply wants lane (i = l % 16, j = l / 16) to hold 8 inputs of
  // tile row i, the same 8 for all i.  Loaded that way an instruction touches 16 rows x 64 bytes --
  // half lines, which streams 12 % slower than whole lines (5.9 against 6.7 TB/s in isolation).
  // So the two fragments of a k-group (64 inputs = 128 bytes of a row) are loaded as two
  // instructions of 8 rows x 128 bytes: load h (h = 0, 1), lane l: row 8 h + l % 8, inputs
  // 8 (l / 8) .. + 7 of the k-group.  Lane (i, j) then holds, of load 0: row i % 8, input block 2 j
  // (i < 8) or 2 j + 1 (i >= 8); of load 1: row 8 + i % 8, the same blocks.  One DPP move per
  // register (rotate the row of 16 lanes by 8, written to half of its lanes) turns the pair into
  //   first operand : row i, block 2 j      = load 0 (i < 8) | load 1 rotated (i >= 8)
  //   second operand: row i, block 2 j + 1  = load 0 rotated (i < 8) | load 1 (i >= 8)
  // and the activations follow: the multiplies of a k-group take input blocks (0, 2, 4, 6) and
  // (1, 3, 5, 7) instead of (0 .. 3) and (4 .. 7) -- any split of the 64 inputs will do as long as
  // both operands use the same one.
  static_assert(kMfmaFrags == 2, "the load pattern pairs the two fragments of a k-group");
  const uint32_t lrow = lane & 7u, lk = (uint32_t)(lane >> 3) * 8u;   // a load's row (+ 8 h) and first input
  uint32_t wq[4][2];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t j = kgpr == 4u ? 0u : (kgpr == 2u ? (uint32_t)q & 1u : (uint32_t)q);
    const uint32_t rt = min(G.my_g + G.rg * j, nrt - 1u);
    wq[q][0] = row_off(rt, lrow);
    wq[q][1] = row_off(rt, 8u + lrow);
  }
  // load h of the k-group at input k of the rows at byte offsets ro: this lane's 8 inputs start at
  // k + lk, or are the row's last 8 when that lies past its end (their staged inputs are zeros)
  auto ld_frag = [&](uint32_t ro, uint32_t k, bool real) {
    const uint32_t off = real ? ro + 2u * min(k + lk, K - 8u) : 0u;   // not real: every lane the matrix' first 16 bytes
    return __builtin_nontemporal_load((const MPK_GLOBAL u32x4*)((const MPK_GLOBAL char*)wbase + off));
  };
  // the pair as loaded -> the two operands (in place)
  auto to_operands = [&](u32x4& l0, u32x4& l1) {
    auto ror8 = [](uint32_t old, uint32_t src, auto bank) {   // lanes of `bank`: src of the lane 8 further in its row of 16
      return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, 0x128, 0xF, decltype(bank)::value, false);
    };
    const u32x4 a = l0, b = l1;
    l0 = u32x4{ror8(a.x, b.x, std::integral_constant<int, 0xC>{}), ror8(a.y, b.y, std::integral_constant<int, 0xC>{}),
               ror8(a.z, b.z, std::integral_constant<int, 0xC>{}), ror8(a.w, b.w, std::integral_constant<int, 0xC>{})};
    l1 = u32x4{ror8(b.x, a.x, std::integral_constant<int, 0x3>{}), ror8(b.y, a.y, std::integral_constant<int, 0x3>{}),
               ror8(b.z, a.z, std::integral_constant<int, 0x3>{}), ror8(b.w, a.w, std::integral_constant<int, 0x3>{})};
  };
  // the wavefront's run of k-groups in chunk c; a chunk takes an even number of round slots
  // (>= 2), so that even slots always use fragment buffer A and odd ones B
  auto chunk_kgs = [&](uint32_t c) { return (min(Kc, K - c * Kc) + KG - 1u) / KG; };
  auto run_lo = [&](uint32_t c) { return G.my_s * chunk_kgs(c) / S; };
  auto run_hi = [&](uint32_t c) { return nrtw ? (G.my_s + 1u) * chunk_kgs(c) / S : 0u; };
  auto slots = [&](uint32_t c) {
    const uint32_t lo = run_lo(c), hi = run_hi(c);
    const uint32_t n = hi > lo ? (hi - lo + kgpr - 1u) / kgpr : 0u;
    return max(2u, (n + 1u) & ~1u);
  };
  // requests the 4 FR kilobytes of round slot (c, i) into buf; buf[FR Q + u] = load u of slot
  // group Q's k-group (rows 8 u .. 8 u + 7 of the tile, see above; two fragments after the
  // exchange in step).  Always that many loads, no branch: the compiler counts the loads in flight statically, and a
  // load that may or may not have been issued makes it wait for everything older than it could
  // be -- in effect for the whole pipeline, every round.  For a slot group that does not exist
  // (past the end of the run, or no row tile) all lanes read the matrix' first 16 bytes instead
  // (one cached line; nobody uses the result).
  auto request_round = [&](u32x4* buf, uint32_t c, uint32_t i) {
    const uint32_t cc = min(c, nchunk - 1u);
    const uint32_t kg0 = run_lo(cc) + i * kgpr, hi = c < nchunk ? run_hi(cc) : 0u;
    const uint32_t k0 = cc * Kc;
    static_for<0, 4>([&](auto Qc) {
      constexpr uint32_t Q = (uint32_t)decltype(Qc)::value;
      const uint32_t kg = kg0 + (Q >> sh);
      const bool ok = kg < hi && (kgpr == 1u ? Q < nrtw : true);
#pragma unroll
      for (int u = 0; u < (int)FR; ++u) buf[FR * Q + u] = ld_frag(wq[Q][u], k0 + kg * KG, ok);
    });
  };
  // RMSNorm gains of a chunk, bf16, copied to LDS behind the staged rows (weights: chunk 0's are
  // requested before the event).  All copies into LDS here go from device memory straight to LDS
  // (no registers): 16 bytes per lane, a wavefront's 64 lanes land side by side.
  uint16_t* gl = (uint16_t*)(xs + (size_t)nb * xstride);   // [Kc]
  auto request_gains = [&](uint32_t c) {
    const uint32_t k0 = c * Kc, klen = min(Kc, K - k0), col = 8u * threadIdx.x;
    if (pro_norm && col < klen)
      __builtin_amdgcn_global_load_lds(as_global((const u32x4*)(gain + k0 + col)), (lds_ptr_t)(gl + wave * 512u), 16, 0, 0);
    // between the end of the row and the end of its last k-group the staged inputs are zeros, and
    // so must the gains be: whatever an earlier workgroup left there may read as NaN, and
    // 0 x NaN is NaN
    if (pro_norm)
      for (uint32_t i = klen + threadIdx.x; i < ((klen + 127u) & ~127u); i += kThreads) gl[i] = 0;
  };
  u32x4 wA[4 * FR], wB[4 * FR];
  const bool preload = !(a.flags & kNoPreloadBit);   // off: the ablation of Section 6.5, Fig. 10
  // Both rounds (16 KB per wavefront) are requested before the event.  A wavefront sees its loads
  // complete in the order it issued them, so whatever is requested now stands between the event
  // and the staged input: more than this measured slower.
  request_gains(0u);
  if (preload) {
    request_round(wA, 0u, 0u);
    asm volatile("; first round requested" ::: "memory");
    request_round(wB, 0u, 1u);
    asm volatile("; second round requested" ::: "memory");
  }
  {
    const uint32_t w = wait_fn();
    if (w != kLinDone) return w;   // aborted or pre-empted: the requested weights are dropped
  }
  trace_mark(a, t, 1);
  if (!preload) {
    request_round(wA, 0u, 0u);
    asm volatile("; first round requested after the event" ::: "memory");
  }
  // Staging: the nb rows of a chunk, 256 inputs (1 KB) per instruction, the instructions dealt
  // round-robin to the wavefronts (16 each for a full chunk), with agent-coherent loads straight
  // into LDS.  What lies between the end of a row and the end of its last k-group is zeroed.
  const uint32_t wide = nb > 8u ? 1u : 0u;
  float rowsum = 0.f;   // lane b: this wavefront's sum of squares of staged row b
  auto stage = [&](uint32_t c) {
    const uint32_t k0 = c * Kc, klen = min(Kc, K - k0), kpad = (klen + 127u) & ~127u;
    if (c) request_gains(c);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t n = wave + 8u * (uint32_t)i;
      const uint32_t b = wide ? n >> 3 : n >> 4, seg = wide ? n & 7u : n & 15u;   // Kc / 256 instructions per row
      if (b < nb && seg * 256u < klen) {
        const uint32_t col = seg * 256u + 4u * (uint32_t)lane;
        if (col < klen)
          __builtin_amdgcn_global_load_lds(as_global((const u32x4*)(src_row(b) + k0 + col)), (lds_ptr_t)(xs + (size_t)b * xstride + seg * 256u), 16, 0, 16);
      }
    }
    if (kpad != klen)
      for (uint32_t i = threadIdx.x; i < nb * (kpad - klen); i += kThreads) xs[(size_t)(i / (kpad - klen)) * xstride + klen + i % (kpad - klen)] = 0.f;
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's copies have landed
  };
  // sums of squares of the staged rows (before the gains), needed only by the epilogue: taken
  // behind the chunk's multiplies by wavefronts 0..3 (rows w, w + 4, ...), which are through their
  // share well before the upper four are (they win the arbitration on their SIMDs), so the pass is
  // off the path from the event to the first multiply and costs nothing at the end either
  auto row_squares = [&](uint32_t c) {
    const uint32_t klen = min(Kc, K - c * Kc);
    for (uint32_t r = wave; r < nb && wave < 4u; r += 4u) {
      float sq = 0.f;
      for (uint32_t col = 4u * (uint32_t)lane; col < klen; col += 256u) {
        const float4 v = *(const float4*)(xs + (size_t)r * xstride + col);
        sq = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, sq))));
      }
      sq = wave_sum_dpp(sq);
      if ((uint32_t)lane == r) rowsum += sq;
    }
  };
  // this lane's staged row and which term its column takes in the first multiply
  const uint32_t xrow = min(PACK == 1 ? frow : (PACK == 2 ? (frow & 7u) : (frow & 3u)), nb - 1u);
  const float* xl = xs + (size_t)xrow * xstride + 2u * fk;   // (operand U of a k-group: input block 2 j + U)
  f32x4 acc[4], acc_lo[4];   // (acc_lo: the lo term's products when PACK == 2)
  // one round slot: multiplies what buf holds for slot (c, i) -- fragment u of every slot group
  // against the three terms of that fragment's inputs, converted once per k-group -- and then
  // requests slot (c2, i2), two ahead, into the same registers
  auto step = [&](u32x4* buf, uint32_t c, uint32_t i, uint32_t c2, uint32_t i2) {
    const uint32_t kg0 = run_lo(c) + i * kgpr, hi = run_hi(c);
    if (kg0 < hi) {
#pragma unroll
      for (int q = 0; q < 4; ++q) to_operands(buf[FR * q], buf[FR * q + 1]);
      static_for<0, (int)FR>([&](auto Uc) {
        constexpr uint32_t U = (uint32_t)decltype(Uc)::value;
        u32x4 p0, p1, p2;   // operands of the first, second, third multiply
        static_for<0, 4>([&](auto Qc) {
          constexpr uint32_t Q = (uint32_t)decltype(Qc)::value;
          const uint32_t kg = kg0 + (Q >> sh);
          const bool rowok = kgpr == 1u ? Q < nrtw : true;
          if (kg < hi && rowok) {
            if (Q == 0u || (Q >> sh) != ((Q - 1u) >> sh)) {   // first slot group of its k-group
              const float* src = xl + kg * KG + U * 8u;
              float4 x0 = *(const float4*)src, x1 = *(const float4*)(src + 4);
              if (pro_norm) {
                const u32x4 gg = *(const u32x4*)(gl + kg * KG + 2u * fk + U * 8u);
                x0.x *= bf16_lo(gg.x); x0.y *= bf16_hi(gg.x); x0.z *= bf16_lo(gg.y); x0.w *= bf16_hi(gg.y);
                x1.x *= bf16_lo(gg.z); x1.y *= bf16_hi(gg.z); x1.z *= bf16_lo(gg.w); x1.w *= bf16_hi(gg.w);
              }
              u32x4 h, m, l;
              split8(x0, x1, &h, &m, &l);
              if (PACK == 1) { p0 = h; p1 = m; p2 = l; }
              if (PACK == 2) { p0 = select4(frow < 8u, h, m); p1 = l; }
              if (PACK == 3) p0 = select4(frow < 4u, h, select4(frow < 8u, m, l));
            }
            const bf16x8 av = __builtin_bit_cast(bf16x8, buf[FR * Q + U]);
            acc[Q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, p0), acc[Q], 0, 0, 0);
            if (PACK == 2) acc_lo[Q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, p1), acc_lo[Q], 0, 0, 0);
            if (PACK == 1) {
              acc[Q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, p1), acc[Q], 0, 0, 0);
              acc[Q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, p2), acc[Q], 0, 0, 0);
            }
          }
        });
      });
    }
    request_round(buf, c2, i2);
  };
  for (uint32_t c = 0; c < nchunk; ++c) {
    if (c) lds_barrier();   // everybody has finished with the previous chunk
    stage(c);
    lds_barrier();
    if (c == 0 && !preload) request_round(wB, 0u, 1u);
    if (c == 0) {
      trace_mark(a, t, 2);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = acc_lo[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const uint32_t ns = slots(c);
    for (uint32_t i = 0; i < ns; i += 2u) {
      const bool wrap = i + 2u >= ns;   // the slots two ahead are the first two of the next chunk
      const uint32_t c2 = wrap ? c + 1u : c, i2 = wrap ? 0u : i + 2u;
      step(wA, c, i, c2, i2);
      step(wB, c, i + 1u, c2, i2 + 1u);
    }
    if (pro_norm) row_squares(c);   // (the chunk is still staged: the next barrier is ahead)
  }
  trace_mark(a, t, 8);
  // ---- the column groups of a packed multiply added up: afterwards column b < nb holds the sum
  if (PACK != 1) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // (a lane's column is its index in its row of 16 lanes: the value 8 / 4 columns up comes
        // by a DPP row shift; columns that get nothing are not results)
        const float v = acc[j][i];
        auto up = [](float x, auto ctrl) {
          return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true));
        };
        if (PACK == 2) acc[j][i] = v + up(v, std::integral_constant<int, 0x108>{}) + acc_lo[j][i];        // hi + mid (8 columns up) + lo
        else acc[j][i] = v + up(v, std::integral_constant<int, 0x104>{}) + up(v, std::integral_constant<int, 0x108>{});   // hi + mid + lo, 4 columns apart
      }
  }
  lds_barrier();   // nobody reads the staged input any more: its space takes the partial tiles
  // ---- partial tiles -> LDS.  part[wave][slot group][row 0..15][col 0..15]
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) part[((wave * 4 + j) * 16 + (lane >> 4) * 4 + i) * 16 + (lane & 15)] = acc[j][i];
  if (pro_norm && lane < 16) ssq[wave * 16 + lane] = rowsum;
  lds_barrier();
  return kLinDone;
}

template <class RowOff, class SrcRow, class Wait>
__device__ __forceinline__ uint32_t mfma_job(const StepArgs& a, const TaskDesc& t, float* lds, float* ssq, const MfmaGeom& G,
                                             const uint16_t* wbase, RowOff row_off, SrcRow src_row, bool pro_norm,
                                             const uint16_t* gain, Wait wait_fn) {
  if (G.nb <= 4u) return mfma_job_packed<3>(a, t, lds, ssq, G, wbase, row_off, src_row, pro_norm, gain, wait_fn);
  if (G.nb <= 8u) return mfma_job_packed<2>(a, t, lds, ssq, G, wbase, row_off, src_row, pro_norm, gain, wait_fn);
  return mfma_job_packed<1>(a, t, lds, ssq, G, wbase, row_off, src_row, pro_norm, gain, wait_fn);
}

// Dot product of weight row r (16-row tile r / 16) with batch column bb from the partial tiles a
// job left in LDS: the row tile's slot groups of slice 0, then those of slice 1, ... added in
// that order.
__device__ __forceinline__ float mfma_dot(const float* part, const MfmaGeom& G, uint32_t r, uint32_t bb) {
  const uint32_t rt = r >> 4, row = r & 15u;
  const uint32_t g = rt % G.rg, j = rt / G.rg;
  const uint32_t n = mfma_group_tiles(G.nrt, G.rg, g);   // row tiles of the wavefronts of group g
  const uint32_t q0 = n >= 3u ? j : (n == 2u ? j : 0u), dq = n >= 3u ? 4u : (n == 2u ? 2u : 1u);
  float v = 0.f;
  for (uint32_t s = 0; s < G.ks; ++s) {
    const uint32_t w = s * G.rg + g;
    for (uint32_t q = q0; q < 4u; q += dq) v += part[(((w * 4u + q) * 16u) + row) * 16u + bb];
  }
  return v;
}

// LDS of a linear task (from the task area): job buffers (mfma_x_floats) | res [residual columns][16] f32
// | ssq [8][16] f32 | 1/rms [16] f32.
template <bool MEGA, class Svc = NoJit>
__device__ __forceinline__ uint32_t linear_task_mfma(const TaskDesc& t, const StepArgs& a, float* lds, int32_t wait_ev,
                                                     uint32_t* s_flag, const Svc& svc = Svc{}) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t K = t.K, nb = t.b1 - t.b0, ncols = t.c1 - t.c0;
  const uint32_t gateup = (t.flags & TF_GATEUP) ? 1u : 0u;
  const uint32_t R = ncols << gateup;            // weight rows of the task ("ring rows")
  const MfmaGeom G = mfma_geom(K, nb, (R + 15u) / 16u, wave);
  float* part = lds;
  float* res_lds = lds + mfma_x_floats(nb);                    // [residual columns][16]
  float* ssq = res_lds + (size_t)a.g->lin_res_rows_max * 16;   // [8][16]
  const uint16_t* W = (const uint16_t*)t.w;
  const uint32_t frow = lane & 15u, fk = (uint32_t)(lane >> 4) * 8u;   // fragment row / input offset
  // split-K task (TF_SPLITK): rows [row0, row0 + ncols) of the matrix, inputs of ONE part; the
  // weight pointer is already advanced to the part, rows are ldw apart
  const bool splitk = t.flags & TF_SPLITK;
  const uint32_t parts = splitk ? (t.p3 & 0xFFu) : 1u, my_part = splitk ? (t.p3 >> 8) : 0u;
  const uint32_t Hs = t.ld_out / parts;              // columns of the real output
  const uint32_t row0 = t.c0 - my_part * Hs, ldw = splitk ? t.p1 : K;
  auto row_off = [&](uint32_t rt, uint32_t row) {       // row: this lane's row of the 16-row tile
    const uint32_t r = min(rt * 16u + row, R - 1u);    // rows past the end repeat the last one
    const uint32_t wrow = gateup ? (row0 + (r >> 1) + ((r & 1u) ? t.p0 : 0u)) : row0 + r;
    return wrow * ldw * 2u;   // bytes; the host checks that a weight matrix stays below 4 GB
  };
  auto src_row = [&](uint32_t b) { return t.in + (size_t)(t.b0 + b) * t.ld_in; };
  const bool pro_norm = t.flags & TF_PRO_NORM;
  auto wait_fn = [&]() -> uint32_t {
    if (wait_ev >= 0) {
      const uint32_t w = linear_wait(a, wait_ev, s_flag, wave, lane, svc);
      if (w != kLinDone) return w;
    }
    // the residual slice of this tile goes out first (tile-local, small): its round trip overlaps the staging
    if ((t.flags & TF_EPI_RESID) && !splitk) {
      for (uint32_t i = threadIdx.x; i < nb * ncols; i += kThreads) {
        uint32_t bb = i / ncols, cc = i % ncols;
        res_lds[cc * 16 + bb] = ld_act(t.in2 + (size_t)(t.b0 + bb) * t.ld_out + t.c0 + cc);
      }
    }
    return kLinDone;
  };
  {
    const uint32_t w = mfma_job(a, t, lds, ssq, G, W, row_off, src_row, pro_norm, (const uint16_t*)t.w2, wait_fn);
    if (w != kLinDone) return w;
  }
  trace_mark(a, t, 3);
  // ---- all wavefronts: add the K slices in order, epilogue, outputs; then the notification
  float* inv_lds = ssq + 8 * 16;   // [16] 1/rms of each batch row
  if (pro_norm) {
    if (threadIdx.x < 16) {
      float ss = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) ss += ssq[w * 16 + threadIdx.x];
      inv_lds[threadIdx.x] = 1.0f / sqrtf(ss / (float)K + t.f0);
    }
    lds_barrier();
  }
  {
    float* outp = (t.flags & TF_OUT_LOGITS) ? a.logits : t.out;
    for (uint32_t i = threadIdx.x; i < ncols * nb; i += kThreads) {
      const uint32_t cc = i / nb, bb = i % nb;
      const float inv = pro_norm ? inv_lds[bb] : 1.0f;
      float v;
      if (gateup) {
        const float gte = mfma_dot(part, G, 2 * cc, bb) * inv, up = mfma_dot(part, G, 2 * cc + 1, bb) * inv;
        v = gte / (1.0f + expf(-gte)) * up;
      } else {
        v = mfma_dot(part, G, cc, bb) * inv;
      }
      if ((t.flags & TF_EPI_RESID) && !splitk) v = res_lds[cc * 16 + bb] + v;
      st_act(outp + (size_t)(t.b0 + bb) * t.ld_out + t.c0 + cc, v);   // split-K: the partial sums of this part
    }
  }
  if (MEGA || splitk) {
    // every wavefront's coherent stores complete before anyone is told
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
  }
  if (splitk) {
    // arrival at the row block's counter now that the partial sums are visible; the last of the
    // `parts` tasks adds the parts in order, and the residual, into the real output -- all
    // wavefronts, one output each, the loads of an output in flight together
    uint32_t* last_flag = (uint32_t*)(ssq + 9 * 16);
    if (threadIdx.x == 0) {
      const uint32_t old = __hip_atomic_fetch_add(as_global(a.g->grp_counters + t.p2), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *last_flag = ((old + 1u) % parts == 0u) ? 1u : 0u;   // every step adds exactly `parts` (also when a captured launch is replayed with its step number frozen)
    }
    lds_barrier();
    if (__builtin_amdgcn_readfirstlane(*last_flag)) {
      float* xout = (float*)t.aux0;
      for (uint32_t i = threadIdx.x; i < ncols * nb; i += kThreads) {
        const uint32_t cc = i / nb, bb = i % nb;
        float v = ld_act(t.in2 + (size_t)(t.b0 + bb) * Hs + row0 + cc);
        float pv[8];
#pragma unroll
        for (uint32_t pp = 0; pp < 8; ++pp) pv[pp] = pp < parts ? ld_act(t.out + (size_t)(t.b0 + bb) * t.ld_out + pp * Hs + row0 + cc) : 0.f;
#pragma unroll
        for (uint32_t pp = 0; pp < 8; ++pp) v += pv[pp];   // parts in ascending order (absent ones add zero)
        st_act(xout + (size_t)(t.b0 + bb) * Hs + row0 + cc, v);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    lds_barrier();
  }
  if (wave == 0) {
    if (MEGA && t.trig_event >= 0) signal_from_wave0(a, t, t.trig_event, lane);
    trace_mark(a, t, 4);
  }
  lds_barrier();   // the partial buffer is reused by the next task
  return kLinDone;
}

// ------------------------------------------------------------------------------ mixture of experts
// Section 6.4: an MoE block is a chain of tasks in the same graph.  `route` turns the router's
// output into the meta-tensor (layout next to moe_meta_words); expert tasks are fixed at compile
// time and use the meta-tensor to split the active experts' weight rows evenly among themselves
// at run time; token rows are gathered while the input is staged (no separate gather step).
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = min(v, (uint32_t)__shfl_xor((int)v, off, 64));
  return v;
}

// One task.  Softmax over all experts in fp32, the top_k largest probabilities (ties: lower expert
// index), renormalised to sum one; ranks of a token's experts are in ascending expert index.
__device__ __forceinline__ void body_moe_route(const TaskDesc& t, const StepArgs& a, float* lds) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t E = t.p0, TK = t.p1, B = t.p2, P = B * TK;
  uint32_t* sel = (uint32_t*)lds;          // [P] expert of pair p
  float* wsel = lds + P;                   // [P] weight of pair p
  uint32_t* cnt = (uint32_t*)(lds + 2 * P);   // [E]
  uint32_t* off = cnt + E;                 // [E]
  uint32_t* tokmask = off + E;             // [E] bit b: token b is routed to the expert (batch <= 16)
  uint32_t* pairof = tokmask + E;          // [E][16] pair index of (expert, token)
  uint32_t* meta = (uint32_t*)t.out;
  constexpr int kPerLane = (int)(kMoeMaxExperts / 64);
  const uint32_t nper = (E + 63u) / 64u;   // experts per lane actually present (uniform)
  for (uint32_t p2 = threadIdx.x; p2 < P; p2 += kThreads) {   // a token whose router output is not finite selects nothing
    sel[p2] = 0xFFFFFFFFu;
    wsel[p2] = 0.f;
  }
  for (uint32_t e = threadIdx.x; e < E; e += kThreads) tokmask[e] = 0u;
  lds_barrier();
  for (uint32_t tok = wave; tok < B; tok += kThreads / 64) {
    float pr[kPerLane];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const uint32_t e = (uint32_t)lane + 64u * i;
      pr[i] = -INFINITY;
      if ((uint32_t)i < nper && e < E) pr[i] = ld_act(t.in + (size_t)tok * t.ld_in + e);
      m = fmaxf(m, pr[i]);
    }
    m = wave_max_dpp(m);
    float l = 0.f;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const uint32_t e = (uint32_t)lane + 64u * i;
      const float lg = pr[i];
      pr[i] = 0.f;
      if ((uint32_t)i < nper && e < E) pr[i] = expf(lg - m);
      l += pr[i];
    }
    l = wave_sum_dpp(l);
#pragma unroll
    for (int i = 0; i < kPerLane; ++i)
      if ((uint32_t)i < nper) pr[i] = pr[i] / l;
    uint32_t taken = 0;   // bit i: this lane's expert lane + 64 i is selected
    for (uint32_t j = 0; j < TK; ++j) {
      float best = -1.f;
      uint32_t best_e = 0xFFFFFFFFu;
#pragma unroll
      for (int i = 0; i < kPerLane; ++i) {
        const uint32_t e = (uint32_t)lane + 64u * i;
        if ((uint32_t)i < nper && e < E && !((taken >> i) & 1u) && pr[i] > best) { best = pr[i]; best_e = e; }   // ascending e: ties keep the lower
      }
      const float wbest = wave_max_dpp(best);
      const uint32_t we = wave_min_u32_dpp(best == wbest ? best_e : 0xFFFFFFFFu);
      if (we != 0xFFFFFFFFu && (we & 63u) == (uint32_t)lane) taken |= 1u << (we >> 6);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) s += ((taken >> i) & 1u) ? pr[i] : 0.f;
    s = wave_sum_dpp(s);
    uint32_t before = 0;   // selected experts with a smaller index, so far
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const bool mine = (taken >> i) & 1u;
      const uint64_t mask = __ballot(mine);
      if (mine) {
        const uint32_t rank = before + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        sel[tok * TK + rank] = (uint32_t)lane + 64u * i;
        wsel[tok * TK + rank] = pr[i] / s;
      }
      before += (uint32_t)__popcll(mask);
    }
  }
  lds_barrier();
  // Per-expert token lists without serial scans: a pair thread sets its token's bit in the
  // expert's mask and leaves its pair index in the expert's row of `pairof`; the expert's list
  // is then its mask's bits in ascending order.
  for (uint32_t p2 = threadIdx.x; p2 < P; p2 += kThreads) {
    const uint32_t e = sel[p2], tok = p2 / TK;
    if (e < E) {
      atomicOr(&tokmask[e], 1u << tok);
      pairof[e * 16u + tok] = p2;
    }
  }
  lds_barrier();
  // offsets and the active list: exclusive scans over the experts by wavefront 0, each lane
  // owning kPerLane consecutive experts
  if (wave == 0) {
    uint32_t c[kPerLane], mine = 0, act = 0, mx = 0;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const uint32_t e = (uint32_t)lane * kPerLane + i;
      c[i] = e < E ? (uint32_t)__popc(tokmask[e]) : 0u;
      mine += c[i];
      act += c[i] ? 1u : 0u;
      mx = max(mx, c[i]);
    }
    uint32_t run = mine, arun = act;   // inclusive scans across lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t v = (uint32_t)__shfl_up((int)run, d, 64), w = (uint32_t)__shfl_up((int)arun, d, 64);
      if (lane >= d) { run += v; arun += w; }
    }
    uint32_t o = run - mine, ai = arun - act;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const uint32_t e = (uint32_t)lane * kPerLane + i;
      if (e < E) {
        cnt[e] = c[i];
        off[e] = o;
        if (c[i]) st_act_u32(meta + 2 + ai++, e);
        o += c[i];
      }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, d, 64));
    if (lane == 63) {
      st_act_u32(meta, arun);
      st_act_u32(meta + 1, mx);
    }
  }
  lds_barrier();
  for (uint32_t e = threadIdx.x; e < E; e += kThreads) {
    st_act_u32(meta + 2 + E + e, cnt[e]);
    st_act_u32(meta + 2 + 2 * E + e, off[e]);
    uint32_t o = off[e], m = tokmask[e];
    while (m) {   // ascending token = ascending pair
      const uint32_t tok = (uint32_t)__ffs((int)m) - 1u;
      m &= m - 1u;
      st_act_u32(meta + 2 + 3 * E + o++, pairof[e * 16u + tok]);
    }
  }
  for (uint32_t p2 = threadIdx.x; p2 < P; p2 += kThreads) {
    st_act_u32(meta + 2 + 3 * E + P + p2, __float_as_uint(wsel[p2]));
    st_act_u32(meta + 2 + 3 * E + 2 * P + p2, sel[p2]);
  }
}

// `ntile` 16-row tiles of one expert's weight matrix, starting at tile `tile0`, times the `ne`
// token rows routed to that expert: a matrix-core job (mfma_job) whose input rows are gathered
// through the expert's pair list while they are staged.  All wavefronts take part; ntile <= 32,
// ne <= 16.
// wait_ev >= 0: the job's inputs exist only once that event is activated (the first job of a
// second-stage expert task, see run_moe_task): it is waited for behind the job's first weight
// requests.  Returns false when the step is being aborted.
__device__ __forceinline__ bool moe_expert_job(const TaskDesc& t, const StepArgs& a, float* lds, const uint16_t* W,
                                               uint32_t tile0, uint32_t ntile, uint32_t ne, const uint32_t* plist,
                                               uint32_t TK, int32_t wait_ev, uint32_t* s_flag) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t K = t.K;
  const uint32_t gateup = (t.flags & TF_GATEUP) ? 1u : 0u;
  const bool pro_norm = t.flags & TF_PRO_NORM;
  const MfmaGeom G = mfma_geom(K, ne, ntile, wave);
  float* part = lds;
  float* ssq = lds + moe_x_floats(a.g->batch);   // [8][16]
  uint32_t* rowidx = (uint32_t*)(ssq + 8 * 16);  // [16] pair of each staged row (= output row)
  uint32_t* rowin = rowidx + 16;                 // [16] input row: gate/up reads the token's row, down the pair's
  if (threadIdx.x < ne) {
    const uint32_t pair = plist[threadIdx.x];   // (the task's copy of the meta-tensor in LDS)
    rowidx[threadIdx.x] = pair;
    rowin[threadIdx.x] = gateup ? pair / TK : pair;
  }
  lds_barrier();
  const uint32_t frow = lane & 15u, fk = (uint32_t)(lane >> 4) * 8u;
  auto row_off = [&](uint32_t rt, uint32_t row) {   // row: this lane's row of the 16-row tile
    const uint32_t r = (tile0 + rt) * 16u + row;    // row of the expert's gate/up-interleaved (or plain) order
    const uint32_t wrow = gateup ? ((r >> 1) + ((r & 1u) ? t.p0 : 0u)) : r;
    return wrow * K * 2u;   // bytes from the expert's first row
  };
  auto src_row = [&](uint32_t b) { return t.in + (size_t)__builtin_amdgcn_readfirstlane(rowin[b]) * t.ld_in; };   // uniform: scalar base addresses
  auto wait_fn = [&]() -> uint32_t {
    if (wait_ev < 0) return kLinDone;
    const uint32_t w = linear_wait(a, wait_ev, s_flag, wave, lane, NoJit{});
    trace_mark(a, t, 1);
    return w;
  };
  if (mfma_job(a, t, lds, ssq, G, W, row_off, src_row, pro_norm, (const uint16_t*)t.w2, wait_fn) != kLinDone) return false;
  const uint32_t ncols = (ntile * 16u) >> gateup, col0 = (tile0 * 16u) >> gateup;
  for (uint32_t i = threadIdx.x; i < ncols * ne; i += kThreads) {
    const uint32_t cc = i / ne, bb = i % ne;
    float inv = 1.0f;
    if (pro_norm) {
      float ss = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) ss += ssq[w * 16 + bb];
      inv = 1.0f / sqrtf(ss / (float)K + t.f0);
    }
    float v;
    if (gateup) {
      const float gte = mfma_dot(part, G, 2 * cc, bb) * inv, up = mfma_dot(part, G, 2 * cc + 1, bb) * inv;
      v = gte / (1.0f + expf(-gte)) * up;
    } else {
      v = mfma_dot(part, G, cc, bb);
    }
    st_act(t.out + (size_t)rowidx[bb] * t.ld_out + col0 + cc, v);
  }
  lds_barrier();   // the next job reuses the buffers
  return true;
}

// Expert task `c0` of `p1`: the active experts' 16-row weight tiles, laid end to end in ascending
// expert order, are dealt to the expert tasks in shares of equal cost (the run-time refinement of
// Section 6.4); a task's share is worked off in jobs of at most 32 tiles that stay inside one expert.
// wait_ev >= 0: the caller has NOT waited for the task's event yet (only for the routing task's,
// so the meta-tensor is this step's); the first job does, behind its first weight requests.
__device__ __forceinline__ bool body_moe_expert(const TaskDesc& t, const StepArgs& a, float* lds, int32_t wait_ev = -1,
                                                uint32_t* s_flag = nullptr) {
  const uint32_t* meta = (const uint32_t*)t.in2;
  const uint32_t E = t.p3 & 0xFFFFu, TK = t.p3 >> 16, NT = t.p1, rows_per_expert = t.p2;
  const uint32_t tiles_per_expert = rows_per_expert / 16u;
  // The part of the meta-tensor an expert task reads -- header, active list, per-expert counts and
  // offsets, pair lists -- comes to LDS in one round trip; looked up in device memory, every job
  // cost three dependent trips (expert, its count and offset, its pairs) before its first weight
  // request could go out.
  const uint32_t P = a.g->batch * TK, MW = 2u + 3u * E + P;
  uint32_t* mlds = (uint32_t*)(lds + moe_x_floats(a.g->batch) + 8 * 16 + 32);   // behind the staged row lists
  for (uint32_t i = threadIdx.x; i < MW; i += kThreads) mlds[i] = ld_relaxed(meta + i);
  lds_barrier();
  const uint32_t n_active = min(__builtin_amdgcn_readfirstlane(mlds[0]), E);
  uint32_t u0, u1;   // this task's share of the tiles: equal in cost, see moe_task_share
  moe_task_share(n_active, tiles_per_expert, NT, t.c0, &u0, &u1);
  while (u0 < u1) {
    const uint32_t ai = u0 / tiles_per_expert, tile0 = u0 % tiles_per_expert;
    const uint32_t ntile = min(min(u1 - u0, tiles_per_expert - tile0), 32u);
    const uint32_t e = min(__builtin_amdgcn_readfirstlane(mlds[2 + ai]), E);   // (E: rejected below; the two reads stay inside the copy)
    const uint32_t ne = __builtin_amdgcn_readfirstlane(mlds[2 + E + min(e, E - 1u)]);
    const uint32_t po = __builtin_amdgcn_readfirstlane(mlds[2 + 2 * E + min(e, E - 1u)]);
    if (e >= E || ne == 0 || ne > 16u || po + ne > P) {   // never index with a damaged meta-tensor
      if (threadIdx.x == 0) report(a, DE_BAD_META, e, ne);
      break;
    }
    const uint16_t* W = (const uint16_t*)t.w + (size_t)e * rows_per_expert * t.K;
    if (!moe_expert_job(t, a, lds, W, tile0, ntile, ne, mlds + 2 + 3 * E + po, TK, wait_ev, s_flag)) return false;
    wait_ev = -1;
    u0 += ntile;
  }
  // (no job ran: the task still ends after its event, like every task)
  if (wait_ev >= 0 && !wait_event(a, wait_ev, s_flag)) return false;
  return true;
}

// out[b][c] = resid[b][c] + sum over the token's experts, in ascending expert index, of
// weight x expert output.
__device__ __forceinline__ void body_moe_combine(const TaskDesc& t, const StepArgs& a) {
  const uint32_t E = t.p0, TK = t.p1, P = a.g->batch * TK, H = t.ld_out;
  const uint32_t* meta = (const uint32_t*)t.aux0;
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    for (uint32_t c = t.c0 + threadIdx.x; c < t.c1; c += kThreads) {
      float acc = 0.f;
      for (uint32_t k = 0; k < TK; ++k) {
        const uint32_t p = b * TK + k;
        const float wk = __uint_as_float(ld_relaxed(meta + 2 + 3 * E + P + p));
        acc = fmaf(wk, ld_act(t.in + (size_t)p * t.ld_in + c), acc);
      }
      st_act(t.out + (size_t)b * H + c, ld_act(t.in2 + (size_t)b * H + c) + acc);
    }
  }
}

// cos and sin of position * inv_freq[i]: the angle is formed and reduced to [-pi, pi] in double.
__device__ __forceinline__ void rope_cs(const StepArgs& a, int32_t pos, uint32_t i, float* c, float* s) {
  double ang = (double)pos * as_global(a.g->inv_freq)[i];
  const double two_pi = 6.283185307179586476925286766559;
  ang -= two_pi * rint(ang / two_pi);
  double sd, cd;
  sincos(ang, &sd, &cd);
  *c = (float)cd;
  *s = (float)sd;
}

// Sum over an aligned group of N adjacent lanes (N a power of two <= 64); every lane gets it.
template <int N>
__device__ __forceinline__ float lane_group_sum(float v) {
#pragma unroll
  for (int off = N / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// T3: rotate q and k heads by the sequence position (half-split pairing), copy v, and append the
// new k and v rows to the cache as bf16.  Angles are evaluated in double precision.
__device__ __forceinline__ void body_rope(const TaskDesc& t, const StepArgs& a) {
  const uint32_t d = a.g->head_dim, half = d / 2, nq = a.g->n_q, nkv = a.g->n_kv;
  const uint32_t s0 = t.c0 / d, s1 = t.c1 / d;
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    int32_t pos = a.positions[b] + (int32_t)a.step;
    if (pos < 0 || (uint32_t)pos >= a.g->max_seq) {
      if (threadIdx.x == 0) report(a, DE_BAD_POSITION, b, (uint32_t)pos);
      continue;
    }
    const float* src = t.in + (size_t)b * t.ld_in;
    float* dst = t.out + (size_t)b * t.ld_out;
    // each thread owns two adjacent rotation pairs (i, i+1) so that cache rows are written as
    // 4-byte (two bf16) coherent stores
    for (uint32_t idx = threadIdx.x; idx < (s1 - s0) * (half / 2); idx += kThreads) {
      uint32_t s = s0 + idx / (half / 2), i = 2 * (idx % (half / 2));
      float2 lo = ld_act2(src + s * d + i), hi = ld_act2(src + s * d + i + half);
      if ((t.flags & TF_QK_NORM) && s < nq + nkv) {
        // RMSNorm over the head first: its half/2 threads are one aligned group of lanes
        float ss = lo.x * lo.x + lo.y * lo.y + hi.x * hi.x + hi.y * hi.y;
        ss = (half / 2 == 32) ? lane_group_sum<32>(ss) : lane_group_sum<16>(ss);
        const float inv = 1.0f / sqrtf(ss / (float)d + t.f0);
        const uint16_t* gn = (const uint16_t*)(s < nq ? t.w : t.w2);
        const uint32_t g0 = *as_global((const uint32_t*)(gn + i)), g1 = *as_global((const uint32_t*)(gn + i + half));
        lo.x *= inv * bf16_lo(g0); lo.y *= inv * bf16_hi(g0);
        hi.x *= inv * bf16_lo(g1); hi.y *= inv * bf16_hi(g1);
      }
      float r[4];   // lo.x, lo.y, hi.x, hi.y after rotation
      if (s < nq + nkv) {
        float u0[2] = {lo.x, lo.y}, u1[2] = {hi.x, hi.y};
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          float c, sn;
          rope_cs(a, pos, i + e, &c, &sn);
          r[e] = u0[e] * c - u1[e] * sn;
          r[2 + e] = u1[e] * c + u0[e] * sn;
        }
      } else {
        r[0] = lo.x; r[1] = lo.y; r[2] = hi.x; r[3] = hi.y;
      }
      st_act(dst + s * d + i, r[0]);
      st_act(dst + s * d + i + 1, r[1]);
      st_act(dst + s * d + i + half, r[2]);
      st_act(dst + s * d + i + half + 1, r[3]);
      if (s >= nq) {
        bool is_k = s < nq + nkv;
        uint32_t g = is_k ? s - nq : s - nq - nkv;
        uint16_t* cache = (uint16_t*)(is_k ? t.aux0 : t.aux1);
        uint16_t* row = cache + (((size_t)b * nkv + g) * a.g->max_seq + (uint32_t)pos) * d;
        st_act_u32((uint32_t*)(row + i), (uint32_t)f32_to_bf16(r[0]) | ((uint32_t)f32_to_bf16(r[1]) << 16));
        st_act_u32((uint32_t*)(row + i + half), (uint32_t)f32_to_bf16(r[2]) | ((uint32_t)f32_to_bf16(r[3]) << 16));
      }
    }
  }
}

// Sum over the LPP (8 or 16) adjacent lanes that share one cache position, with DPP lane
// permutations (register-to-register, no LDS round trip); every lane gets the sum.
template <int LPP>
__device__ __forceinline__ float group_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // lane ^ 1
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // lane ^ 2
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // mirror in 8
  if (LPP == 16)
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // mirror in 16
  return v;
}

// Rounds of cache rows the running-softmax attention body keeps in registers (requested ahead of
// their use), by the kernel's batch class nb (0: the generic kernels) and query heads per KV head.
// Batch 1: chunks are a few rounds long and the task is a chain of latencies -- as many rounds as
// the running state of the heads leaves registers for, so that a whole chunk is requested before
// the event.  Matrix-core batch classes: chunks are tens of rounds long and all 256 workers stream
// at once; three rounds in flight per wavefront measured fastest (8B shape at batch 8: 5.29 ms per
// step against 5.30 / 5.36 / 5.36 / 5.52 with 2 / 4 / 6 / 8; the mixture-of-experts shape at batch
// 16: 15.0 against 15.5 / 15.4 with 2 / 4) -- what is in flight beyond that only lengthens the
// queue in front of everybody's next request.
constexpr int attn_depth(int nb, int grp) { return nb >= 5 ? 3 : (grp <= 4 ? 8 : 4); }
constexpr bool attn_streams(int nb) { return nb >= 5; }

__device__ __forceinline__ void unpack8(const u32x4& w, float (&f)[8]) {   // 8 bf16 -> fp32
  f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x); f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
  f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z); f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

// 16 bytes of a cache row of an earlier step.  Contiguous cache: a plain streaming load (the row's
// lines were never read in this launch before they were written, see the attention body).  Paged
// cache: a page that one request gave back may be handed to another within the same launch, so a
// compute unit may still hold lines of the page's previous life -- in a launch that runs several
// steps every row is read with agent-scope loads, which do not hit such lines; a launch of one
// step cannot see a page change owners (the serving task runs before any row is read), so there
// the streaming load is as good as on the contiguous cache.
template <bool PAGED>
__device__ __forceinline__ u32x4 ld_cache_row(const StepArgs& a, const uint16_t* p) {
  if constexpr (PAGED) {
    if (a.flags & kOneStepBit) return ld_stream16(p);
    return ld_row16_coherent(p);
  } else {
    return ld_stream16(p);
  }
}

// Position of sequence b in this step.  positions[] is the host's and stays as written for the
// whole launch (tasks add the step number) -- except in a serving launch, where the serving task
// rewrites it at the start of every step: then it holds the step's own positions and is read with
// coherent loads, after the serving task's event.
template <bool PAGED>
__device__ __forceinline__ int32_t step_position(const StepArgs& a, uint32_t b) {
  if (PAGED && (a.flags & kServeBit)) return (int32_t)ld_relaxed((const uint32_t*)a.positions + b);
  return a.positions[b] + (int32_t)a.step;
}

// T4, short chunks: the same task when a chunk never exceeds kAttnRounds rounds (8 x 32 = 256 cache
// positions at head_dim 128): all of its K and V rows are requested before the event wait and
// stay in registers, scores are formed once, one chunk-wide maximum, one exp per score.  Fewer
// instructions than the running-softmax body below; the decoder at batch 1 spends its attention
// phase on latency, not bandwidth, so that is what counts there.
// Layout of the work: D/8 adjacent lanes share one position (16 bytes of the row each), a
// wavefront covers 64/(D/8) positions per round, the 8 wavefronts of the workgroup take rounds
// of 8 x that many positions; kAttnRounds rounds fit in registers and the compiler picks the chunk
// count so that a chunk never exceeds them.
// Cache rows of earlier steps are immutable during a step, so the task requests its K and V rows
// BEFORE it waits for its dependent event; only the query (and the row appended this step)
// arrive later.  Scores, probabilities and the running sums stay in registers.
constexpr int kAttnRounds = 8;

template <int D, int GRP, bool PAGED = false>
__device__ __forceinline__ bool body_attn_partial_regs(const TaskDesc& t, const StepArgs& a, float* lds,
                                                  int32_t wait_ev, uint32_t* s_flag) {
  constexpr uint32_t d = D, grp = GRP, LPP = D / 8, PPW = 64 / LPP, NW = kThreads / 64;
  constexpr uint32_t stride = NW * PPW, per = grp * (d + 2);
  constexpr uint32_t WS = d + 4;   // row of one partial in LDS: output, max, sum; 16-byte aligned rows
  const uint32_t nq = a.g->n_q, nkv = a.g->n_kv, C = t.p1;
  const uint32_t b = t.b0, u = t.c0 / per, g = u / C, c = u % C;
  // (paged cache: positions and page table are this step's once the serving task has run -- see
  // the running-softmax body below)
  if (PAGED && wait_ev >= 0 && a.g->serve_event >= 0 && !wait_event(a, a.g->serve_event, s_flag)) return false;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* qs = lds;                       // [grp][d]
  float* wpart = qs + grp * d;           // [NW * PPW][grp][WS]: partial output and sum per position slot
  uint32_t* flag = (uint32_t*)(wpart + stride * grp * WS);    // then [16..) the maxima exchange
  float* outp = t.out + (size_t)b * t.ld_out + t.c0;
  const int32_t pos = step_position<PAGED>(a, b);    // written by the host before the launch (or by the serving task)
  const bool bad_pos = pos < 0 || (uint32_t)pos >= a.g->max_seq;
  const uint32_t len = bad_pos ? 0u : (uint32_t)pos + 1;
  const uint32_t t0 = (uint32_t)((uint64_t)c * len / C), t1 = (uint32_t)((uint64_t)(c + 1) * len / C);
  const uint32_t n = t1 - t0;
  const uint16_t* Kb = (const uint16_t*)t.aux0 + (PAGED ? (size_t)0 : (((size_t)b * nkv + g) * a.g->max_seq + t0) * d);
  const uint16_t* Vb = (const uint16_t*)t.aux1 + (PAGED ? (size_t)0 : (((size_t)b * nkv + g) * a.g->max_seq + t0) * d);
  // paged: the chunk's page numbers, staged in LDS (behind the maxima exchange)
  const uint32_t pshift = PAGED ? a.g->page_shift : 0u;
  const uint32_t pg0 = t0 >> pshift;
  uint32_t* pgs = flag + 48;
  bool bad_page = false;
  if constexpr (PAGED) {
    const uint32_t* ptab = (const uint32_t*)a.g->page_table + (size_t)b * (a.g->max_seq >> pshift);
    const uint32_t npg = n ? ((t1 - 1u) >> pshift) - pg0 + 1u : 0u;
    for (uint32_t i = threadIdx.x; i < npg; i += kThreads) {
      uint32_t pg = ld_relaxed(ptab + pg0 + i);
      if (pg >= a.g->kv_pages) { bad_page = true; pg = 0; }
      pgs[i] = pg;
    }
    __syncthreads();
    if (bad_page) report(a, DE_BAD_PAGE, b, t0);   // (its rows come from page 0 instead: wrong, but in bounds)
  }
  auto row_off = [&](uint32_t i) -> size_t {   // element offset of row i of the chunk from Kb / Vb
    if constexpr (PAGED) {
      const uint32_t r = t0 + i;
      return ((((size_t)pgs[(r >> pshift) - pg0] * nkv + g) << pshift) + (r & ((1u << pshift) - 1u))) * d;
    } else {
      return (size_t)i * d;
    }
  };
  const uint32_t sub = lane % LPP, slot = lane / LPP;
  const uint32_t i_first = wave * PPW + slot;
  const uint32_t n_rounds = (n + stride - 1) / stride;
  // ---- pre-load: K and V rows of earlier steps
  u32x4 kreg[kAttnRounds], vreg[kAttnRounds];
  auto load_rows = [&]() {
#pragma unroll
    for (int r = 0; r < kAttnRounds; ++r) {
      const uint32_t i = i_first + r * stride;
      kreg[r] = u32x4{0, 0, 0, 0};
      vreg[r] = u32x4{0, 0, 0, 0};
      if (i < n && t0 + i != (uint32_t)pos) {
        const size_t off = row_off(i);
        kreg[r] = ld_cache_row<PAGED>(a, Kb + off + sub * 8);
        vreg[r] = ld_cache_row<PAGED>(a, Vb + off + sub * 8);
      }
    }
  };
  const bool preload = !(a.flags & kNoPreloadBit);
  if (preload) {
    load_rows();
    asm volatile("; cache rows requested" ::: "memory");
  }
  // the rotation angles depend on the position alone: worked out (in double precision) before the
  // event, off the critical path from the QKV projection to the O projection.  A thread's first
  // query element, and the two key pairs of the threads that append the new row.
  float pre_cs = 1.f, pre_sn = 0.f, pre_c0 = 1.f, pre_s0 = 0.f, pre_c1 = 1.f, pre_s1 = 0.f;
  if (t.flags & TF_ROPE_FUSED) {
    if (threadIdx.x < grp * (d / 2)) rope_cs(a, pos, threadIdx.x % (d / 2), &pre_cs, &pre_sn);
    const uint32_t ik = kThreads - 1 - threadIdx.x;
    if (c == C - 1 && ik < d / 4) {
      rope_cs(a, pos, 2 * ik, &pre_c0, &pre_s0);
      rope_cs(a, pos, 2 * ik + 1, &pre_c1, &pre_s1);
    }
  }
  if (wait_ev >= 0 && !wait_event(a, wait_ev, s_flag)) return false;
  trace_mark(a, t, 1);
  if (!preload) {
    load_rows();
    asm volatile("; cache rows requested after the event" ::: "memory");
  }
  if (bad_pos || n_rounds > (uint32_t)kAttnRounds) {
    if (threadIdx.x == 0) report(a, DE_BAD_POSITION, b, (uint32_t)pos);
    for (uint32_t i = threadIdx.x; i < per; i += kThreads) st_act(outp + i, ((i % (d + 2)) == d) ? -INFINITY : 0.f);
    return true;
  }
  const float* qsrc = t.in + (size_t)b * t.ld_in + (size_t)g * grp * d;
  if (t.flags & TF_ROPE_FUSED) {
    // the input is the raw QKV projection: rotate the group's query heads here; the task of the
    // last chunk also rotates this step's key, and appends key and value to the cache
    constexpr uint32_t half = d / 2;
    const bool qk_norm = t.flags & TF_QK_NORM;
    for (uint32_t i = threadIdx.x; i < grp * half; i += kThreads) {
      uint32_t j = i / half, e = i % half;
      float u0 = ld_act(qsrc + j * d + e), u1 = ld_act(qsrc + j * d + e + half), cs, sn;
      if (qk_norm) {   // RMSNorm over the head: its `half` threads are one aligned group of lanes
        const float inv = 1.0f / sqrtf(lane_group_sum<(int)half>(u0 * u0 + u1 * u1) / (float)d + t.f0);
        const uint16_t* gq = (const uint16_t*)t.w;
        u0 *= inv * bf16_to_f32(as_global(gq)[e]);
        u1 *= inv * bf16_to_f32(as_global(gq)[e + half]);
      }
      if (i < kThreads) { cs = pre_cs; sn = pre_sn; }
      else rope_cs(a, pos, e, &cs, &sn);
      qs[j * d + e] = u0 * cs - u1 * sn;
      qs[j * d + e + half] = u1 * cs + u0 * sn;
    }
    if (c == C - 1) {
      const float* ksrc = t.in + (size_t)b * t.ld_in + (size_t)(nq + g) * d;
      const float* vsrc = t.in + (size_t)b * t.ld_in + (size_t)(nq + nkv + g) * d;
      uint16_t *krow, *vrow;
      if constexpr (PAGED) {
        const size_t off = row_off((uint32_t)pos - t0);
        krow = const_cast<uint16_t*>(Kb) + off;
        vrow = const_cast<uint16_t*>(Vb) + off;
      } else {
        krow = (uint16_t*)t.aux0 + (((size_t)b * nkv + g) * a.g->max_seq + (uint32_t)pos) * d;
        vrow = (uint16_t*)t.aux1 + (((size_t)b * nkv + g) * a.g->max_seq + (uint32_t)pos) * d;
      }
      // threads from the top of the workgroup, so that they do not also rotate query pairs
      for (uint32_t i = kThreads - 1 - threadIdx.x; i < half / 2 + half; i += kThreads) {
        if (i < half / 2) {   // two adjacent rotation pairs of the key
          uint32_t e = 2 * i;
          float2 lo = ld_act2(ksrc + e), hi = ld_act2(ksrc + e + half);
          if (qk_norm) {   // the key's half/2 threads: one aligned group of lanes at the top of the workgroup
            const float ss = lane_group_sum<(int)(half / 2)>(lo.x * lo.x + lo.y * lo.y + hi.x * hi.x + hi.y * hi.y);
            const float inv = 1.0f / sqrtf(ss / (float)d + t.f0);
            const uint16_t* gk = (const uint16_t*)t.w2;
            const uint32_t g0 = *as_global((const uint32_t*)(gk + e)), g1 = *as_global((const uint32_t*)(gk + e + half));
            lo.x *= inv * bf16_lo(g0); lo.y *= inv * bf16_hi(g0);
            hi.x *= inv * bf16_lo(g1); hi.y *= inv * bf16_hi(g1);
          }
          const float c0 = pre_c0, s0 = pre_s0, c1 = pre_c1, s1 = pre_s1;   // (i < half / 2 <= kThreads: the first pass)
          float r0 = lo.x * c0 - hi.x * s0, r1 = lo.y * c1 - hi.y * s1;
          float r2 = hi.x * c0 + lo.x * s0, r3 = hi.y * c1 + lo.y * s1;
          st_act_u32((uint32_t*)(krow + e), (uint32_t)f32_to_bf16(r0) | ((uint32_t)f32_to_bf16(r1) << 16));
          st_act_u32((uint32_t*)(krow + e + half), (uint32_t)f32_to_bf16(r2) | ((uint32_t)f32_to_bf16(r3) << 16));
        } else {              // two adjacent value elements
          uint32_t e = 2 * (i - half / 2);
          float2 v2 = ld_act2(vsrc + e);
          st_act_u32((uint32_t*)(vrow + e), (uint32_t)f32_to_bf16(v2.x) | ((uint32_t)f32_to_bf16(v2.y) << 16));
        }
      }
      // the appended row is read back below with coherent loads: the stores must have completed
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
  } else {
    for (uint32_t i = threadIdx.x; i < grp * d; i += kThreads) qs[i] = ld_act(qsrc + i);
  }
  __syncthreads();
  trace_mark(a, t, 2);
  // The row appended during this step is read with coherent loads (it was written after the
  // pre-load, by this or another workgroup); it can only be the last position of the last chunk.
  if (c == C - 1) {
    const uint32_t i_new = n - 1;
#pragma unroll
    for (int r = 0; r < kAttnRounds; ++r) {
      if (i_first + r * stride == i_new) {
        const size_t off = row_off(i_new);
        kreg[r] = ld_row16_coherent(Kb + off + sub * 8);
        vreg[r] = ld_row16_coherent(Vb + off + sub * 8);
      }
    }
  }
  // ---- per block of HB heads (bounds the register footprint): scores, softmax statistics and
  // P.V, all in registers; sreg[r][j] belongs to position i_first + r * stride, head jb + j
  constexpr int HB = GRP < 4 ? GRP : 4;
  const float inv_sqrt_d = 1.0f / sqrtf((float)d);
  // The body is bound by vector instructions, not by memory (two wavefronts per SIMD, about a
  // thousand instructions each for a full chunk): rounds the chunk does not reach are skipped.
  // The count is the same in every lane (it comes from positions[b]); say so to the compiler.
  const uint32_t n_rounds_u = __builtin_amdgcn_readfirstlane(n_rounds);
  float* mxch = wpart + stride * grp * WS + 16;   // [NW][HB] maxima exchange
  // scores are kept times log2(e): the probabilities are then one v_exp_f32 each
  const float score_scale = inv_sqrt_d * 1.44269504088896341f;
  float m_all[GRP];
#pragma unroll 1
  for (int jb = 0; jb < GRP; jb += HB) {
    float q[HB][8];
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      const float4* qp = (const float4*)(qs + (jb + j) * d + sub * 8);
      float4 q0 = qp[0], q1 = qp[1];
      q[j][0] = q0.x; q[j][1] = q0.y; q[j][2] = q0.z; q[j][3] = q0.w;
      q[j][4] = q1.x; q[j][5] = q1.y; q[j][6] = q1.z; q[j][7] = q1.w;
    }
    float sreg[kAttnRounds][HB];
    float mloc[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) mloc[j] = -INFINITY;
#pragma unroll
    for (int r = 0; r < kAttnRounds; ++r) {
      if ((uint32_t)r >= n_rounds_u) continue;   // (uniform) rounds past the chunk: nothing to do
      const bool valid = i_first + r * stride < n;
      const u32x4 kv = kreg[r];
      const float k8[8] = {bf16_lo(kv.x), bf16_hi(kv.x), bf16_lo(kv.y), bf16_hi(kv.y),
                           bf16_lo(kv.z), bf16_hi(kv.z), bf16_lo(kv.w), bf16_hi(kv.w)};
#pragma unroll
      for (int j = 0; j < HB; ++j) {
        float sv = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sv = fmaf(k8[e], q[j][e], sv);
        sv = group_sum<LPP>(sv) * score_scale;
        sreg[r][j] = valid ? sv : -INFINITY;
        mloc[j] = fmaxf(mloc[j], sreg[r][j]);
      }
    }
    // chunk maximum per head: across position slots, then across wavefronts
#pragma unroll
    for (int j = 0; j < HB; ++j) {
#pragma unroll
      for (uint32_t off = LPP; off < 64; off <<= 1) mloc[j] = fmaxf(mloc[j], __shfl_xor(mloc[j], off, 64));
      if (lane == 0) mxch[wave * HB + j] = mloc[j];
    }
    __syncthreads();
    float m[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      float v = mxch[j];
#pragma unroll
      for (uint32_t w = 1; w < NW; ++w) v = fmaxf(v, mxch[w * HB + j]);
      m[j] = v;
      m_all[jb + j] = v * 0.693147180559945309f;   // the partial's maximum is stored in natural units
    }
    // ---- probabilities and P.V
    float acc[HB][8], lsum[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      lsum[j] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[j][e] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < kAttnRounds; ++r) {
      if ((uint32_t)r >= n_rounds_u) continue;
      const u32x4 vv = vreg[r];
      const float v8[8] = {bf16_lo(vv.x), bf16_hi(vv.x), bf16_lo(vv.y), bf16_hi(vv.y),
                           bf16_lo(vv.z), bf16_hi(vv.z), bf16_lo(vv.w), bf16_hi(vv.w)};
#pragma unroll
      for (int j = 0; j < HB; ++j) {
        const float p = (sreg[r][j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sreg[r][j] - m[j]);
        lsum[j] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[j][e] = fmaf(p, v8[e], acc[j][e]);
      }
    }
    // every position slot's partial goes to LDS as it is (two 16-byte stores per head); the
    // slots are added up below, by the threads that write the result.  (Adding them with lane
    // shuffles first cost 4 instructions per value here, where instructions are what is scarce.)
#pragma unroll
    for (int j = 0; j < HB; ++j) {
      float4* wp = (float4*)(wpart + ((size_t)(wave * PPW + slot) * grp + jb + j) * WS + sub * 8);
      wp[0] = make_float4(acc[j][0], acc[j][1], acc[j][2], acc[j][3]);
      wp[1] = make_float4(acc[j][4], acc[j][5], acc[j][6], acc[j][7]);
      // every lane of a position group holds the same p: one of them stores the sum
      if (sub == 0) wpart[((size_t)(wave * PPW + slot) * grp + jb + j) * WS + d + 1] = lsum[j];
    }
    __syncthreads();   // also protects mxch before the next block
  }
  trace_mark(a, t, 10);
  for (uint32_t i = threadIdx.x; i < grp * (d + 2); i += kThreads) {
    const uint32_t j = i / (d + 2), dim = i % (d + 2);
    float sv;
    if (dim == d) {
      sv = m_all[0];
#pragma unroll
      for (int jj = 1; jj < GRP; ++jj) sv = (j == (uint32_t)jj) ? m_all[jj] : sv;
    } else {
      sv = 0.f;
#pragma unroll
      for (uint32_t w = 0; w < stride; ++w) sv += wpart[((size_t)w * grp + j) * WS + dim];
    }
    st_act(outp + i, sv);
  }
  trace_mark(a, t, 11);
  if (t.flags & TF_ATTN_MERGE) {
    // Arrival counter of (layer, sequence, KV head): the chunk task that arrives last sees all C
    // partials complete and merges them (log-sum-exp, one pass with running maximum) into the
    // attention output.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t* cnt = a.g->grp_counters + t.p2 + b * nkv + g;
      uint32_t old = __hip_atomic_fetch_add(as_global(cnt), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *flag = ((old + 1u) % C == 0u) ? 1u : 0u;   // every step adds exactly C
    }
    __syncthreads();
    if (*flag) {
      const float* part = t.out + (size_t)b * t.ld_out + (size_t)g * C * per;
      float* o = const_cast<float*>(t.in2) + (size_t)b * nq * d + (size_t)g * grp * d;
      for (uint32_t i = threadIdx.x; i < grp * d; i += kThreads) {
        uint32_t j = i / d, dim = i % d;
        float M = -INFINITY, L = 0.f, acc_o = 0.f;
        for (uint32_t c0 = 0; c0 < C; c0 += 8) {   // 24 coherent loads in flight: one round trip for 8 chunks
          float mm[8], ll[8], oo[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            if (c0 + k < C) {
              const float* pp = part + ((size_t)(c0 + k) * grp + j) * (d + 2);
              mm[k] = ld_act(pp + d);
              ll[k] = ld_act(pp + d + 1);
              oo[k] = ld_act(pp + dim);
            } else {
              mm[k] = -INFINITY; ll[k] = 0.f; oo[k] = 0.f;
            }
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            float Mn = fmaxf(M, mm[k]);
            if (Mn == -INFINITY) continue;   // empty chunks only so far
            float sc_old = expf(M - Mn), sc_new = expf(mm[k] - Mn);
            L = L * sc_old + ll[k] * sc_new;
            acc_o = acc_o * sc_old + oo[k] * sc_new;
            M = Mn;
          }
        }
        st_act(o + i, acc_o / L);
      }
    }
  }
  return true;
}

// TF_ATTN_BALANCE: the batch x C chunk tasks of a KV head, numbered v = row x C + chunk, are dealt
// to the sequences in proportion to their lengths, every sequence at least one: sequence b gets
// 1 + floor((batch x C - batch) x len_b / total) tasks, and what is left over (fewer than batch)
// goes, one at a time, to the sequence whose chunks are longest at that moment (lowest index on
// ties).  A pure function of the positions, worked out by every wavefront for itself (lane b <
// batch holds sequence b; batch <= 16).  Returns the sequence of task v, the task's chunk number
// there, the sequence's chunk count and its first task.
template <bool PAGED>
__device__ __forceinline__ void attn_deal(const StepArgs& a, uint32_t C, uint32_t v, uint32_t* seq, uint32_t* chunk,
                                          uint32_t* chunks, uint32_t* first) {
  const uint32_t B = a.g->batch, li = threadIdx.x & 15u;
  uint32_t w = 0;
  if (li < B) {
    const int32_t pos = step_position<PAGED>(a, li);
    w = (pos >= 0 && (uint32_t)pos < a.g->max_seq) ? (uint32_t)pos + 1u : 1u;   // (a bad position is reported by its tasks)
  }
  auto row_sum = [&](uint32_t x) {   // over the 16 lanes of the row, in every lane
#pragma unroll
    for (uint32_t off = 1; off < 16; off <<= 1) x += (uint32_t)__shfl_xor((int)x, off, 16);
    return x;
  };
  const uint32_t total = row_sum(w);
  uint32_t cnt = li < B ? 1u + (uint32_t)((uint64_t)(B * C - B) * w / total) : 0u;
  const uint32_t left = B * C - row_sum(cnt);   // uniform, < B
  for (uint32_t r = 0; r < left; ++r) {
    const float len = li < B ? (float)w / (float)cnt : -1.f;   // current chunk length of the sequence
    float mx = len;
#pragma unroll
    for (uint32_t off = 1; off < 16; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 16));
    const uint32_t who = (uint32_t)__ballot(len == mx) & 0xFFFFu;   // (the wavefront's first 16 lanes)
    if (li == (uint32_t)__builtin_ctz(who)) ++cnt;
  }
  uint32_t end = cnt;   // inclusive prefix sum: first task after the sequence
#pragma unroll
  for (uint32_t off = 1; off < 16; off <<= 1) {
    const uint32_t o = (uint32_t)__shfl_up((int)end, off, 16);
    if (li >= off) end += o;
  }
  const uint32_t start = end - cnt;
  const uint32_t mask = (uint32_t)__ballot(li < B && start <= v) & 0xFFFFu;
  const uint32_t bsel = 31u - (uint32_t)__builtin_clz(mask);                  // start of sequence 0 is 0 <= v
  *seq = bsel;
  *first = (uint32_t)__builtin_amdgcn_readlane((int)start, bsel);
  *chunks = (uint32_t)__builtin_amdgcn_readlane((int)cnt, bsel);
  *chunk = v - *first;
}

// T4: split-KV decode attention for one (sequence, KV head, chunk).  Chunk c of C covers cache
// rows [c*len/C, (c+1)*len/C) with len = position + 1, so the last chunk holds the new row.
// Output per query head of the group: sum_t exp(s_t - m) V_t (D floats), m, l = sum_t exp(s_t - m).
// Layout of the work: D/8 adjacent lanes share one position (16 bytes of the row each), a
// wavefront covers 64/(D/8) positions per round, the wavefronts of the workgroup take rounds of
// (wavefronts x that many) positions.  Every lane group keeps a running maximum, sum and output
// per query head (online softmax), so a chunk may be of any length and no barrier is needed until
// the end, where the lane groups of a wavefront are combined with lane shuffles and the
// wavefronts through LDS.
// Cache rows of earlier steps are immutable during a step, so the task requests its first
// kAttnPre rounds of K and V rows BEFORE it waits for its dependent event; only the query (and the
// row appended this step) arrive later.  Later rounds are requested a batch at a time.
// These early reads are plain non-temporal loads.  In a multi-token launch they include the row
// another workgroup appended in the PREVIOUS step of the same launch; that is safe because (1) the
// row was written with coherent stores that completed before its task notified, and this worker
// has since waited for an event downstream of that notification (a step's first tasks wait for
// the previous step's terminal event), and (2) no cache can hold an older copy of the row's
// lines: a row fills whole 128-byte lines of its own and is never read before it is written (the
// row at the current position is excluded from the early reads and fetched coherently).
// The caller in turn must not change rows below a sequence's position while a launch runs.
// PAGED (TF_KV_PAGED; paper Section 6.1, paged attention): the cache is a pool of pages
// [kv_pages][n_kv][page][D] per layer and row r of sequence b is row r % page of page
// page_table[b][r / page].  The table (and, in a serving launch, positions[]) belong to THIS step
// only once the serving task has run, so the task first waits for that task's event -- activated
// at the very start of the step, long before the task's own event -- and only then deals the chunk
// tasks, looks up its pages and requests its rows.  Table entries are read with coherent loads
// (one per row and lane group; the lookups of a batch of rounds travel together).  An entry
// outside the pool is reported and replaced by page 0: no address ever leaves the pool.
template <int D, int GRP, bool PAGED = false, int NB = 0>
__device__ __forceinline__ bool body_attn_partial(const TaskDesc& t, const StepArgs& a, float* lds,
                                                  int32_t wait_ev, uint32_t* s_flag) {
  constexpr uint32_t d = D, grp = GRP, LPP = D / 8, PPW = 64 / LPP, NW = kThreads / 64;
  constexpr uint32_t stride = NW * PPW, per = grp * (d + 2);
  const uint32_t nq = a.g->n_q, nkv = a.g->n_kv, Cs = t.p1;
  const uint32_t bs = t.b0, u = t.c0 / per, g = u / Cs;   // the task's own row: where its partial result goes
  if (PAGED && wait_ev >= 0 && a.g->serve_event >= 0 && !wait_event(a, a.g->serve_event, s_flag)) return false;
  // sequence, chunk and chunk count the task works on, first task of that sequence
  uint32_t b = bs, c = u % Cs, C = Cs, v0 = bs * Cs;
  if (t.flags & TF_ATTN_BALANCE) attn_deal<PAGED>(a, Cs, bs * Cs + c, &b, &c, &C, &v0);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* qs = lds;                       // [grp][d]
  float* wpart = qs + grp * d;           // [NW][grp][d + 2]: partial output, max, sum per wavefront
  uint32_t* flag = (uint32_t*)(wpart + NW * grp * (d + 2));
  float* outp = t.out + (size_t)bs * t.ld_out + t.c0;
  const int32_t pos = step_position<PAGED>(a, b);    // written by the host before the launch (or by the serving task)
  const bool bad_pos = pos < 0 || (uint32_t)pos >= a.g->max_seq;
  const uint32_t len = bad_pos ? 0u : (uint32_t)pos + 1;
  const uint32_t t0 = (uint32_t)((uint64_t)c * len / C), t1 = (uint32_t)((uint64_t)(c + 1) * len / C);
  const uint32_t n = t1 - t0;
  // contiguous cache: the chunk's first row; paged: the layer's pools
  const uint16_t* Kb = (const uint16_t*)t.aux0 + (PAGED ? (size_t)0 : (((size_t)b * nkv + g) * a.g->max_seq + t0) * d);
  const uint16_t* Vb = (const uint16_t*)t.aux1 + (PAGED ? (size_t)0 : (((size_t)b * nkv + g) * a.g->max_seq + t0) * d);
  // paged: the page numbers of the chunk's rows go to LDS first (one coherent load per page, all in
  // flight together), so that a row's address costs an LDS read, not a trip to memory
  const uint32_t pshift = PAGED ? a.g->page_shift : 0u;
  const uint32_t pg0 = t0 >> pshift;
  uint32_t* pgs = flag + 16;
  bool bad_page = false;
  if constexpr (PAGED) {
    const uint32_t* ptab = (const uint32_t*)a.g->page_table + (size_t)b * (a.g->max_seq >> pshift);
    const uint32_t npg = n ? ((t1 - 1u) >> pshift) - pg0 + 1u : 0u;
    for (uint32_t i = threadIdx.x; i < npg; i += kThreads) {
      uint32_t pg = ld_relaxed(ptab + pg0 + i);
      if (pg >= a.g->kv_pages) { bad_page = true; pg = 0; }
      pgs[i] = pg;
    }
    __syncthreads();
  }
  // element offset of row i of the chunk (row t0 + i of the sequence) from Kb / Vb
  auto row_off = [&](uint32_t i) -> size_t {
    if constexpr (PAGED) {
      const uint32_t r = t0 + i;
      return ((((size_t)pgs[(r >> pshift) - pg0] * nkv + g) << pshift) + (r & ((1u << pshift) - 1u))) * d;
    } else {
      return (size_t)i * d;
    }
  };
  const uint32_t sub = lane % LPP, slot = lane / LPP;
  const uint32_t i_first = wave * PPW + slot;
  const uint32_t n_rounds = (n + stride - 1) / stride;
  constexpr int kAttnPre = attn_depth(NB, GRP);   // rounds held in registers at a time
  constexpr bool STREAM = attn_streams(NB);         // which of the two request schedules below
  // the row appended this step, if in this chunk: it is written after the early reads (by this or
  // another workgroup), so it is never among them and is fetched with coherent loads when its turn
  // comes (STREAM: after all the rounds)
  const uint32_t i_new = (!bad_pos && c == C - 1) ? n - 1 : 0xFFFFFFFFu;
  // ---- STREAM: K and V rows of round `rnd` into register pair r.  Always two loads, no branch around
  // them: the compiler counts the loads in flight statically, and a load that may or may not have
  // been issued makes every later wait a wait for everything.  A position the chunk does not have
  // (or the appended row) reads the chunk's last row of an earlier step again -- this compute
  // unit's own line, already on its way or cached -- and nobody uses the result; a chunk with no
  // such row reads 16 bytes of the task array (immutable).
  u32x4 kreg[kAttnPre], vreg[kAttnPre];
  const uint16_t* nothing = (const uint16_t*)a.tasks;
  const uint32_t n_old = n - (i_new != 0xFFFFFFFFu ? 1u : 0u);   // rows of earlier steps in the chunk
  // (`coherent`: which kind of load a paged cache needs in this launch, see ld_cache_row -- a
  // compile-time choice here, made once per task by the callers: a branch around the load would
  // spoil the count just the same)
  auto request_round = [&](auto coherent, int r, uint32_t rnd) {
    const uint32_t i = min(i_first + rnd * stride, n_old - 1u);
    const bool ok = n_old != 0u;
    const size_t off = ok ? row_off(i) + sub * 8 : (size_t)0;
    const uint16_t *kp = ok ? Kb + off : nothing, *vp = ok ? Vb + off : nothing;
    kreg[r] = decltype(coherent)::value ? ld_row16_coherent(kp) : ld_stream16(kp);
    vreg[r] = decltype(coherent)::value ? ld_row16_coherent(vp) : ld_stream16(vp);
  };
  const bool coherent_rows = PAGED && !(a.flags & kOneStepBit);
  // ---- pre-load: the first rounds (never the row appended this step)
  auto load_rows = [&]() {
    if constexpr (STREAM) {
      if (coherent_rows) {
#pragma unroll
        for (int r = 0; r < kAttnPre; ++r) request_round(std::true_type{}, r, (uint32_t)r);
      } else {
#pragma unroll
        for (int r = 0; r < kAttnPre; ++r) request_round(std::false_type{}, r, (uint32_t)r);
      }
    } else {
#pragma unroll
      for (int r = 0; r < kAttnPre; ++r) {
        const uint32_t i = i_first + r * stride;
        kreg[r] = u32x4{0, 0, 0, 0};
        vreg[r] = u32x4{0, 0, 0, 0};
        if (i < n && i != i_new) {
          const size_t off = row_off(i);
          kreg[r] = ld_cache_row<PAGED>(a, Kb + off + sub * 8);
          vreg[r] = ld_cache_row<PAGED>(a, Vb + off + sub * 8);
        }
      }
    }
  };
  const bool preload = !(a.flags & kNoPreloadBit);
  if (preload) {
    load_rows();
    asm volatile("; cache rows requested" ::: "memory");
  }
  // the rotation angles depend on the position alone: worked out (in double precision) before the
  // event, off the critical path from the QKV projection to the O projection.  A thread's first
  // query element, and the two key pairs of the threads that append the new row.
  float pre_cs = 1.f, pre_sn = 0.f, pre_c0 = 1.f, pre_s0 = 0.f, pre_c1 = 1.f, pre_s1 = 0.f;
  if (t.flags & TF_ROPE_FUSED) {
    if (threadIdx.x < grp * (d / 2)) rope_cs(a, pos, threadIdx.x % (d / 2), &pre_cs, &pre_sn);
    const uint32_t ik = kThreads - 1 - threadIdx.x;
    if (c == C - 1 && ik < d / 4) {
      rope_cs(a, pos, 2 * ik, &pre_c0, &pre_s0);
      rope_cs(a, pos, 2 * ik + 1, &pre_c1, &pre_s1);
    }
  }
  if (wait_ev >= 0 && !wait_event(a, wait_ev, s_flag)) return false;
  trace_mark(a, t, 1);
  if (!preload) {
    load_rows();
    asm volatile("; cache rows requested after the event" ::: "memory");
  }
  if (bad_pos) {
    if (threadIdx.x == 0) report(a, DE_BAD_POSITION, b, (uint32_t)pos);
    for (uint32_t i = threadIdx.x; i < per; i += kThreads) st_act(outp + i, ((i % (d + 2)) == d) ? -INFINITY : 0.f);
    return true;
  }
  const float* qsrc = t.in + (size_t)b * t.ld_in + (size_t)g * grp * d;
  if (t.flags & TF_ROPE_FUSED) {
    // the input is the raw QKV projection: rotate the group's query heads here; the task of the
    // last chunk also rotates this step's key, and appends key and value to the cache
    constexpr uint32_t half = d / 2;
    const bool qk_norm = t.flags & TF_QK_NORM;
    for (uint32_t i = threadIdx.x; i < grp * half; i += kThreads) {
      uint32_t j = i / half, e = i % half;
      float u0 = ld_act(qsrc + j * d + e), u1 = ld_act(qsrc + j * d + e + half), cs, sn;
      if (qk_norm) {   // RMSNorm over the head: its `half` threads are one aligned group of lanes
        const float inv = 1.0f / sqrtf(lane_group_sum<(int)half>(u0 * u0 + u1 * u1) / (float)d + t.f0);
        const uint16_t* gq = (const uint16_t*)t.w;
        u0 *= inv * bf16_to_f32(as_global(gq)[e]);
        u1 *= inv * bf16_to_f32(as_global(gq)[e + half]);
      }
      if (i < kThreads) { cs = pre_cs; sn = pre_sn; }
      else rope_cs(a, pos, e, &cs, &sn);
      qs[j * d + e] = u0 * cs - u1 * sn;
      qs[j * d + e + half] = u1 * cs + u0 * sn;
    }
    if (c == C - 1) {
      const float* ksrc = t.in + (size_t)b * t.ld_in + (size_t)(nq + g) * d;
      const float* vsrc = t.in + (size_t)b * t.ld_in + (size_t)(nq + nkv + g) * d;
      uint16_t *krow, *vrow;
      if constexpr (PAGED) {
        const size_t off = row_off((uint32_t)pos - t0);
        krow = const_cast<uint16_t*>(Kb) + off;
        vrow = const_cast<uint16_t*>(Vb) + off;
      } else {
        krow = (uint16_t*)t.aux0 + (((size_t)b * nkv + g) * a.g->max_seq + (uint32_t)pos) * d;
        vrow = (uint16_t*)t.aux1 + (((size_t)b * nkv + g) * a.g->max_seq + (uint32_t)pos) * d;
      }
      // threads from the top of the workgroup, so that they do not also rotate query pairs
      for (uint32_t i = kThreads - 1 - threadIdx.x; i < half / 2 + half; i += kThreads) {
        if (i < half / 2) {   // two adjacent rotation pairs of the key
          uint32_t e = 2 * i;
          float2 lo = ld_act2(ksrc + e), hi = ld_act2(ksrc + e + half);
          if (qk_norm) {   // the key's half/2 threads: one aligned group of lanes at the top of the workgroup
            const float ss = lane_group_sum<(int)(half / 2)>(lo.x * lo.x + lo.y * lo.y + hi.x * hi.x + hi.y * hi.y);
            const float inv = 1.0f / sqrtf(ss / (float)d + t.f0);
            const uint16_t* gk = (const uint16_t*)t.w2;
            const uint32_t g0 = *as_global((const uint32_t*)(gk + e)), g1 = *as_global((const uint32_t*)(gk + e + half));
            lo.x *= inv * bf16_lo(g0); lo.y *= inv * bf16_hi(g0);
            hi.x *= inv * bf16_lo(g1); hi.y *= inv * bf16_hi(g1);
          }
          const float c0 = pre_c0, s0 = pre_s0, c1 = pre_c1, s1 = pre_s1;   // (i < half / 2 <= kThreads: the first pass)
          float r0 = lo.x * c0 - hi.x * s0, r1 = lo.y * c1 - hi.y * s1;
          float r2 = hi.x * c0 + lo.x * s0, r3 = hi.y * c1 + lo.y * s1;
          st_act_u32((uint32_t*)(krow + e), (uint32_t)f32_to_bf16(r0) | ((uint32_t)f32_to_bf16(r1) << 16));
          st_act_u32((uint32_t*)(krow + e + half), (uint32_t)f32_to_bf16(r2) | ((uint32_t)f32_to_bf16(r3) << 16));
        } else {              // two adjacent value elements
          uint32_t e = 2 * (i - half / 2);
          float2 v2 = ld_act2(vsrc + e);
          st_act_u32((uint32_t*)(vrow + e), (uint32_t)f32_to_bf16(v2.x) | ((uint32_t)f32_to_bf16(v2.y) << 16));
        }
      }
      // the appended row is read back below with coherent loads: the stores must have completed
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
  } else {
    for (uint32_t i = threadIdx.x; i < grp * d; i += kThreads) qs[i] = ld_act(qsrc + i);
  }
  __syncthreads();
  trace_mark(a, t, 2);
  // ---- running softmax per lane group and query head.  Scores and maxima are kept times
  // log2(e), folded into the query, so that every probability and rescale is one v_exp_f32 (the
  // body is bound by vector instructions at 4 and 8 query heads per KV head).
  const float inv_sqrt_d = 1.44269504088896341f / sqrtf((float)d);
  float q[GRP][8], m[GRP], l[GRP], acc[GRP][8];
#pragma unroll
  for (int j = 0; j < GRP; ++j) {
    const float4* qp = (const float4*)(qs + j * d + sub * 8);
    const float4 q0 = qp[0], q1 = qp[1];
    q[j][0] = q0.x * inv_sqrt_d; q[j][1] = q0.y * inv_sqrt_d; q[j][2] = q0.z * inv_sqrt_d; q[j][3] = q0.w * inv_sqrt_d;
    q[j][4] = q1.x * inv_sqrt_d; q[j][5] = q1.y * inv_sqrt_d; q[j][6] = q1.z * inv_sqrt_d; q[j][7] = q1.w * inv_sqrt_d;
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[j][e] = 0.f;
  }
  // one position per lane group: score, running maximum, probability, P.V
  auto consume = [&](const float (&k8)[8], const float (&v8)[8], bool valid) {
#pragma unroll
    for (int j = 0; j < GRP; ++j) {
      float sv = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) sv = fmaf(k8[e], q[j][e], sv);
      sv = group_sum<LPP>(sv);
      if (valid) {
        if (sv > m[j]) {   // a new maximum (rare after the first positions): rescale the running state
          const float sc = __builtin_amdgcn_exp2f(m[j] - sv);   // 2^(-inf) = 0 on the first position
          l[j] *= sc;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[j][e] *= sc;
          m[j] = sv;
        }
        const float p = __builtin_amdgcn_exp2f(sv - m[j]);
        l[j] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[j][e] = fmaf(p, v8[e], acc[j][e]);
      }
    }
  };
  if constexpr (STREAM) {
    // Long chunks, every worker streaming: kAttnPre rounds live in registers; a pair is requested
    // again, kAttnPre rounds ahead, as soon as it has been used, so that all but one of them are
    // in flight while one is multiplied.
    auto rounds = [&](auto coherent) {
      for (uint32_t r0 = 0; r0 < n_rounds; r0 += kAttnPre) {
#pragma unroll
        for (int r = 0; r < kAttnPre; ++r) {
          const uint32_t i = i_first + (r0 + r) * stride;
          float k8[8], v8[8];
          unpack8(kreg[r], k8);
          unpack8(vreg[r], v8);
          request_round(coherent, r, r0 + r + kAttnPre);   // (behind the unpacking: the pair's registers are free)
          consume(k8, v8, i < n && i != i_new);
        }
      }
    };
    if (coherent_rows) rounds(std::true_type{});
    else rounds(std::false_type{});
    if (i_new != 0xFFFFFFFFu) {   // (uniform) the appended row: the lane group its position falls to
      const size_t off = row_off(i_new) + sub * 8;
      float k8[8], v8[8];
      unpack8(ld_row16_coherent(Kb + off), k8);
      unpack8(ld_row16_coherent(Vb + off), v8);
      consume(k8, v8, i_new % stride == i_first);
    }
  } else {
    // Short chunks (a few rounds, most often all of them requested before the event): a batch of
    // rounds lives in registers; its first half is requested again (for the next batch) as soon
    // as it has been used, the second half at the end of the batch, and only when the chunk goes
    // on -- a chunk that fits the registers issues no further request at all.
    constexpr int kHalf = kAttnPre / 2;
    auto request_next = [&](uint32_t r0, auto first_half) {
      constexpr int lo = decltype(first_half)::value ? 0 : kHalf, hi = decltype(first_half)::value ? kHalf : kAttnPre;
      if (r0 + kAttnPre < n_rounds) {
#pragma unroll
        for (int r = lo; r < hi; ++r) {
          const uint32_t i = i_first + (r0 + kAttnPre + r) * stride;
          if (i < n && i != i_new) {
            const size_t off = row_off(i);
            kreg[r] = ld_cache_row<PAGED>(a, Kb + off + sub * 8);
            vreg[r] = ld_cache_row<PAGED>(a, Vb + off + sub * 8);
          }
        }
      }
    };
    for (uint32_t r0 = 0; r0 < n_rounds; r0 += kAttnPre) {
#pragma unroll
      for (int r = 0; r < kAttnPre; ++r) {
        if (r == kHalf) request_next(r0, std::true_type{});
        const uint32_t i = i_first + (r0 + r) * stride;
        if (i == i_new) {
          // written after the pre-load, by this or another workgroup: coherent loads
          const size_t off = row_off(i);
          kreg[r] = ld_row16_coherent(Kb + off + sub * 8);
          vreg[r] = ld_row16_coherent(Vb + off + sub * 8);
        }
        float k8[8], v8[8];
        unpack8(kreg[r], k8);
        unpack8(vreg[r], v8);
        consume(k8, v8, i < n);
      }
      request_next(r0, std::false_type{});
    }
  }
  if (PAGED && bad_page) report(a, DE_BAD_PAGE, b, t0);   // (the rows came from page 0 instead: wrong, but in bounds)
  // ---- combine the lane groups of the wavefront, then the wavefronts
#pragma unroll
  for (int j = 0; j < GRP; ++j) {
#pragma unroll
    for (uint32_t off = LPP; off < 64; off <<= 1) {
      const float mo = __shfl_xor(m[j], off, 64), lo2 = __shfl_xor(l[j], off, 64);
      const float mn = fmaxf(m[j], mo);
      const float s0 = (m[j] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[j] - mn), s1 = (mo == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mo - mn);
      l[j] = l[j] * s0 + lo2 * s1;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[j][e] = acc[j][e] * s0 + __shfl_xor(acc[j][e], off, 64) * s1;
      m[j] = mn;
    }
    if (slot == 0) {
      float* wp = wpart + ((size_t)wave * grp + j) * (d + 2);
#pragma unroll
      for (int e = 0; e < 8; ++e) wp[sub * 8 + e] = acc[j][e];
      if (sub == 0) {
        wp[d] = m[j] * 0.693147180559945309f;   // back to natural units for the merges
        wp[d + 1] = l[j];
      }
    }
  }
  __syncthreads();
  trace_mark(a, t, 10);
  for (uint32_t i = threadIdx.x; i < grp * (d + 2); i += kThreads) {
    const uint32_t j = i / (d + 2), dim = i % (d + 2);
    float M = -INFINITY;
#pragma unroll
    for (uint32_t w = 0; w < NW; ++w) M = fmaxf(M, wpart[((size_t)w * grp + j) * (d + 2) + d]);
    float sv;
    if (dim == d) {
      sv = M;
    } else {
      sv = 0.f;
      const uint32_t src = (dim == d + 1) ? d + 1 : dim;
#pragma unroll
      for (uint32_t w = 0; w < NW; ++w) {
        const float mw = wpart[((size_t)w * grp + j) * (d + 2) + d];
        if (mw != -INFINITY) sv += wpart[((size_t)w * grp + j) * (d + 2) + src] * expf(mw - M);
      }
    }
    st_act(outp + i, sv);
  }
  trace_mark(a, t, 11);
  if (t.flags & TF_ATTN_MERGE) {
    // Arrival counter of (layer, sequence, KV head): the chunk task that arrives last sees all C
    // partials complete and merges them (log-sum-exp, one pass with running maximum) into the
    // attention output.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t* cnt = a.g->grp_counters + t.p2 + b * nkv + g;
      uint32_t old = __hip_atomic_fetch_add(as_global(cnt), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (t.flags & TF_ATTN_BALANCE) {
        // the count changes with the lengths from step to step: the last arrival puts the counter
        // back to zero (nobody else touches it before the next step's attention tasks)
        *flag = (old + 1u == C) ? 1u : 0u;
        if (old + 1u == C) st_act_u32(cnt, 0u);
      } else {
        *flag = ((old + 1u) % C == 0u) ? 1u : 0u;   // every step adds exactly C
      }
    }
    __syncthreads();
    if (*flag) {
      // chunk k of the sequence is the partial result of task v0 + k, in that task's own slot
      auto part_of = [&](uint32_t k) {
        const uint32_t v = v0 + k;
        return t.out + (size_t)(v / Cs) * t.ld_out + (size_t)(g * Cs + v % Cs) * per;
      };
      float* o = const_cast<float*>(t.in2) + (size_t)b * nq * d + (size_t)g * grp * d;
      for (uint32_t i = threadIdx.x; i < grp * d; i += kThreads) {
        uint32_t j = i / d, dim = i % d;
        float M = -INFINITY, L = 0.f, acc_o = 0.f;
        for (uint32_t c0 = 0; c0 < C; c0 += 8) {   // 24 coherent loads in flight: one round trip for 8 chunks
          float mm[8], ll[8], oo[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            if (c0 + k < C) {
              const float* pp = part_of(c0 + k) + (size_t)j * (d + 2);
              mm[k] = ld_act(pp + d);
              ll[k] = ld_act(pp + d + 1);
              oo[k] = ld_act(pp + dim);
            } else {
              mm[k] = -INFINITY; ll[k] = 0.f; oo[k] = 0.f;
            }
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            float Mn = fmaxf(M, mm[k]);
            if (Mn == -INFINITY) continue;   // empty chunks only so far
            float sc_old = expf(M - Mn), sc_new = expf(mm[k] - Mn);
            L = L * sc_old + ll[k] * sc_new;
            acc_o = acc_o * sc_old + oo[k] * sc_new;
            M = Mn;
          }
        }
        st_act(o + i, acc_o / L);
      }
    }
  }
  return true;
}

// T5: merge the chunk partials of each query head with the log-sum-exp rule.
__device__ __forceinline__ void body_attn_merge(const TaskDesc& t, const StepArgs& a) {
  const uint32_t d = a.g->head_dim, grp = a.g->n_q / a.g->n_kv, C = t.p1;
  const uint32_t h0 = t.c0 / d, h1 = t.c1 / d;
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    const float* part = t.in + (size_t)b * t.ld_in;
    float* out = t.out + (size_t)b * t.ld_out;
    for (uint32_t idx = threadIdx.x; idx < (h1 - h0) * d; idx += kThreads) {
      uint32_t h = h0 + idx / d, dim = idx % d, g = h / grp, j = h % grp;
      float M = -INFINITY;
      for (uint32_t c = 0; c < C; ++c) M = fmaxf(M, ld_act(part + ((size_t)(g * C + c) * grp + j) * (d + 2) + d));
      float L = 0.f, o = 0.f;
      for (uint32_t c = 0; c < C; ++c) {
        const float* p = part + ((size_t)(g * C + c) * grp + j) * (d + 2);
        float wgt = expf(ld_act(p + d) - M);   // exp(-inf) = 0 for empty chunks
        L = fmaf(wgt, ld_act(p + d + 1), L);
        o = fmaf(wgt, ld_act(p + dim), o);
      }
      st_act(out + h * d + dim, o / L);
    }
  }
}

__device__ __forceinline__ void body_add(const TaskDesc& t) {
  const uint32_t nc = t.c1 - t.c0;
  for (uint32_t b = t.b0; b < t.b1; ++b)
    for (uint32_t i = threadIdx.x; i < nc; i += kThreads) {
      size_t o = (size_t)b * t.ld_out + t.c0 + i;
      st_act(t.out + o, ld_act(t.in + o) + ld_act(t.in2 + o));
    }
}

__device__ __forceinline__ void body_swiglu(const TaskDesc& t) {
  const uint32_t nc = t.c1 - t.c0, F = t.p0;
  for (uint32_t b = t.b0; b < t.b1; ++b)
    for (uint32_t i = threadIdx.x; i < nc; i += kThreads) {
      const float* gu = t.in + (size_t)b * t.ld_in;
      float gte = ld_act(gu + t.c0 + i), up = ld_act(gu + F + t.c0 + i);
      st_act(t.out + (size_t)b * t.ld_out + t.c0 + i, gte / (1.0f + expf(-gte)) * up);
    }
}

// Greedy sampling: the index of the largest logit of a sequence, lowest index on ties.  T tasks
// per sequence (t.p1): task j scans logits [V j / T, V (j+1) / T) -- it depends only on the LM-head
// tasks that produce them -- and leaves (largest value, its index) in its pair of the output row;
// the task of a sequence that arrives last (arrival counter t.p2 + sequence, T arrivals per step)
// picks the token from the T pairs.  The token goes to token_ids[b] for the next step's embedding
// task (and to tokens_out); the last step of a launch also advances positions[b].  Optionally
// keeps a copy of the logits.
__device__ __forceinline__ void body_argmax(const TaskDesc& t, const StepArgs& a, float* lds) {
  const int lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t V = t.K, B = a.g->batch, T = t.p1, j = t.c0 / 2u;
  const uint32_t q = V / T, r = V % T;
  const uint32_t v0 = j * q + min(j, r), v1 = (j + 1u) * q + min(j + 1u, r);   // the even split of V into T shares
  float* vmax = lds;                          // [8]
  uint32_t* imax = (uint32_t*)(lds + 8);      // [8]
  for (uint32_t b = t.b0; b < t.b1; ++b) {
    const float* row = a.logits + (size_t)b * V;
    float* const logits_all = a.g->logits_all;
    int32_t* const tokens_out = a.g->tokens_out;
    float* copy = logits_all ? logits_all + ((size_t)a.step * B + b) * V : nullptr;
    float best = -INFINITY;
    uint32_t best_i = 0xFFFFFFFFu;
    // One workgroup reads its share with coherent loads: what counts is how many of them are in
    // flight (one at a time, the row of a 152k vocabulary took about 150 us -- 5 % of a batch-1
    // step of the 8B shape).  32 per thread are requested before the first is looked at.
    constexpr int kInFlight = 32;
    for (uint32_t i0 = v0 + threadIdx.x; i0 < v1; i0 += kThreads * kInFlight) {   // ascending per thread: keeps the first maximum
      float v[kInFlight];
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const uint32_t i = i0 + (uint32_t)u * kThreads;
        v[u] = i < v1 ? ld_act(row + i) : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        const uint32_t i = i0 + (uint32_t)u * kThreads;
        if (i < v1) {
          if (copy) as_global(copy)[i] = v[u];
          if (v[u] > best || best_i == 0xFFFFFFFFu) { best = v[u]; best_i = i; }
        }
      }
    }
    const float wbest = wave_max(best);
    const uint32_t wi = wave_min_u32(best == wbest ? best_i : 0xFFFFFFFFu);
    if (lane == 0) { vmax[wave] = wbest; imax[wave] = wi; }
    lds_barrier();
    if (threadIdx.x == 0) {
      float m = vmax[0];
      uint32_t mi = imax[0];
      for (uint32_t w = 1; w < kThreads / 64; ++w)
        if (vmax[w] > m || (vmax[w] == m && imax[w] < mi)) { m = vmax[w]; mi = imax[w]; }
      bool pick = true;
      if (T > 1u) {
        float* pairs = t.out + (size_t)b * t.ld_out;
        st_act(pairs + 2u * j, m);
        st_act_u32((uint32_t*)pairs + 2u * j + 1u, mi);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the pair is in place before the arrival counts
        uint32_t* cnt = a.g->grp_counters + t.p2 + b;
        const uint32_t old = __hip_atomic_fetch_add(as_global(cnt), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        pick = (old + 1u) % T == 0u;   // every step adds exactly T
        if (pick) {
          float pm[32];
          uint32_t pi[32];
#pragma unroll
          for (uint32_t k = 0; k < 32u; ++k) {
            if (k < T) { pm[k] = ld_act(pairs + 2u * k); pi[k] = ld_relaxed((const uint32_t*)pairs + 2u * k + 1u); }
          }
          m = pm[0];
          mi = pi[0];
#pragma unroll
          for (uint32_t k = 1; k < 32u; ++k)
            if (k < T && pm[k] > m) { m = pm[k]; mi = pi[k]; }   // shares ascend with k: the first maximum stays
        }
      }
      if (pick) {
        if (mi >= V) mi = 0;   // logits that are not numbers: keep the token in range
        st_act_u32((uint32_t*)const_cast<int32_t*>(a.token_ids) + b, mi);
        if (tokens_out) st_act_u32((uint32_t*)tokens_out + (size_t)a.step * B + b, mi);
        if ((uint32_t)a.step + 1u == a.n_steps && !(a.flags & kServeBit))   // (a serving launch: the serving task keeps the positions)
          st_act_u32((uint32_t*)const_cast<int32_t*>(a.positions) + b, (uint32_t)(a.positions[b] + (int32_t)a.n_steps));
      }
    }
    lds_barrier();
  }
}

// The task on the start event of a serving graph (paper Section 6.1: the scheduler prepares a new
// decoding iteration by (1) removing completed requests, (2) admitting newly arrived requests and
// (3) updating the per-request KV-cache metadata; "this logic executes as a single task").  The
// paper fixes no policy; this one is the library's contract (mpk_serve_* in the public header):
//   (1) a slot whose request still has prompt tokens is fed the next one (the sampled token is
//       ignored: prompts go through the decode path a token per iteration); otherwise the sampled
//       token is the request's next output, and the request is finished on the end-of-sequence
//       token or with max_new tokens.  Finished slots, in ascending order, push their pages onto
//       the free stack in page-table order.
//   (2) idle slots, in ascending order, take the queued requests in arrival order, each only if
//       the pages it can ever need, ceil((prompt + max_new - 1) / page), are free and not promised
//       to running requests; the first request that does not fit ends admission (no overtaking).
//   (3) a running slot whose position is at a page boundary pops a page (ascending slot order);
//       an idle slot computes on token 0 at position 0 in its own page (page number = slot).
// One wavefront, lane b = slot b (batch <= 16): every slot's state is loaded and stored once, the
// sequential decisions (stack positions, admission) are prefix counts over lanes, so the task is
// a handful of memory round trips however many slots change.  All state is read and written with
// agent-scope accesses: attention tasks on other compute units read the tables in the same step.
__device__ __forceinline__ void body_serve(const StepArgs& a) {
  const ServeDev* Sp = a.g->serve;
  if (threadIdx.x >= 64 || Sp == nullptr) return;
  const ServeDev sv = *Sp;
  const uint32_t lane = threadIdx.x, B = a.g->batch, n_pages = a.g->kv_pages;
  const uint32_t shift = sv.page_shift, ps_mask = (1u << shift) - 1u;
  const bool mine = lane < B;
  const uint64_t below = (1ull << lane) - 1ull;
  uint32_t* tok_io = (uint32_t*)const_cast<int32_t*>(a.token_ids);
  uint32_t* pos_io = (uint32_t*)const_cast<int32_t*>(a.positions);
  int32_t req = mine ? (int32_t)ld_relaxed((const uint32_t*)sv.slot_req + lane) : -1;
  uint32_t pos = mine ? ld_relaxed((const uint32_t*)sv.slot_pos + lane) : 0u;
  uint32_t held = mine ? ld_relaxed((const uint32_t*)sv.slot_held + lane) : 0u;
  const uint32_t sampled = mine ? ld_relaxed(tok_io + lane) : 0u;
  uint32_t n_free = __builtin_amdgcn_readfirstlane(ld_relaxed(sv.scalars + kServeNFree));
  uint32_t promised = __builtin_amdgcn_readfirstlane(ld_relaxed(sv.scalars + kServePromised));
  uint32_t q_head = __builtin_amdgcn_readfirstlane(ld_relaxed(sv.scalars + kServeQHead));
  const uint32_t q_tail = __builtin_amdgcn_readfirstlane(ld_relaxed(sv.scalars + kServeQTail));
  auto pages_of = [&](uint32_t plen, uint32_t max_new) { return (plen + max_new - 1u + ps_mask) >> shift; };
  // ---- (1) completed requests leave
  uint32_t nxt = 0, need = 0;
  bool done = false, produced = false;
  if (req >= 0) {
    const uint32_t plen = ld_relaxed(sv.req_len + 2 * (size_t)req), max_new = ld_relaxed(sv.req_len + 2 * (size_t)req + 1);
    need = pages_of(plen, max_new);
    const uint32_t cached = pos + 1u;
    if (cached < plen) {
      nxt = ld_relaxed((const uint32_t*)sv.req_prompt + (size_t)req * sv.max_prompt + cached);
    } else {
      uint32_t n_out = ld_relaxed(sv.req_state + 2 * (size_t)req + 1);
      if (n_out < sv.max_new) st_act_u32((uint32_t*)sv.req_out + (size_t)req * sv.max_new + n_out, sampled);
      ++n_out;
      st_act_u32(sv.req_state + 2 * (size_t)req + 1, n_out);
      nxt = sampled;
      produced = true;
      done = (int32_t)sampled == sv.eos || n_out >= max_new;
    }
    pos = cached;
  }
  const uint32_t n_produced = (uint32_t)__builtin_popcountll(__ballot(produced));
  const uint32_t n_done = (uint32_t)__builtin_popcountll(__ballot(done));
  for (uint64_t retiring = __ballot(done); retiring; retiring &= retiring - 1ull) {
    const uint32_t b = (uint32_t)__builtin_ctzll(retiring);
    const uint32_t hb = (uint32_t)__builtin_amdgcn_readlane((int)held, (int)b);
    const uint32_t nb = (uint32_t)__builtin_amdgcn_readlane((int)need, (int)b);
    uint32_t* row = (uint32_t*)sv.table + (size_t)b * sv.max_blocks;
    for (uint32_t i = lane; i < hb && i < sv.max_blocks; i += 64u) {
      const uint32_t pg = ld_relaxed(row + i);
      if (n_free + i < n_pages) st_act_u32((uint32_t*)sv.free_stack + n_free + i, pg);
      st_act_u32(row + i, i == 0u ? b : 0xFFFFFFFFu);   // the idle slot's own page; the rest: none
    }
    n_free += hb;
    promised -= nb - hb;
  }
  if (done) {
    st_act_u32(sv.req_state + 2 * (size_t)req, 2u);
    req = -1;
    held = 0;
    pos = 0;
  }
  // ---- (1b) the running requests close ranks: in order, to the lowest slots (a slot is metadata
  // only, the rows stay in their pages), so that the graph of a smaller batch size can serve them
  {
    const uint64_t run_mask = __ballot(mine && req >= 0);
    const uint32_t n_run = (uint32_t)__builtin_popcountll(run_mask);
    if (run_mask != (1ull << n_run) - 1ull) {   // (uniform) there are gaps
      uint32_t my_src = lane, k = 0;
      for (uint64_t m = run_mask; m; m &= m - 1ull, ++k) {
        const uint32_t src = (uint32_t)__builtin_ctzll(m);
        if (lane == k) my_src = src;
        if (src == k) continue;
        // page-table row src -> row k (k < src; rows below k are final, rows above src untouched so far)
        const uint32_t hb = (uint32_t)__builtin_amdgcn_readlane((int)held, (int)src);
        uint32_t* from = (uint32_t*)sv.table + (size_t)src * sv.max_blocks;
        uint32_t* to = (uint32_t*)sv.table + (size_t)k * sv.max_blocks;
        for (uint32_t i = lane; i < sv.max_blocks; i += 64u) {
          const uint32_t v = i < hb ? ld_relaxed(from + i) : 0xFFFFFFFFu;
          st_act_u32(to + i, v);
          st_act_u32(from + i, i == 0u ? src : 0xFFFFFFFFu);   // vacated (a later move may fill it again)
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the next move may read what this one wrote
      }
      const int src_lane = (int)my_src;
      const int32_t req_m = __shfl(req, src_lane, 64);
      const uint32_t pos_m = (uint32_t)__shfl((int)pos, src_lane, 64), held_m = (uint32_t)__shfl((int)held, src_lane, 64);
      const uint32_t nxt_m = (uint32_t)__shfl((int)nxt, src_lane, 64);
      const bool keep = lane < n_run;
      req = keep ? req_m : -1;
      pos = keep ? pos_m : 0u;
      held = keep ? held_m : 0u;
      nxt = keep ? nxt_m : 0u;
    }
  }
  // the pages pushed above may be popped below, by other lanes: the stores must have completed
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  // ---- (2) arrivals enter, in order, while their pages are there
  const bool idle = mine && req < 0;
  const uint64_t idle_mask = __ballot(idle);
  const uint32_t n_idle = (uint32_t)__builtin_popcountll(idle_mask);
  uint32_t c_plen = 0, c_new = 0;   // lane i < 16: the request that is i-th in the queue
  if (lane < 16u && q_head + lane < q_tail && q_head + lane < sv.max_requests) {
    c_plen = ld_relaxed(sv.req_len + 2 * (size_t)(q_head + lane));
    c_new = ld_relaxed(sv.req_len + 2 * (size_t)(q_head + lane) + 1);
  }
  const uint32_t c_need = pages_of(c_plen, c_new);
  uint32_t n_admit = 0;
  for (uint32_t k = 0; k < n_idle; ++k) {
    if (q_head + k >= q_tail || q_head + k >= sv.max_requests) break;
    const uint32_t nd = (uint32_t)__builtin_amdgcn_readlane((int)c_need, (int)k);
    if (n_free - promised < nd) break;
    promised += nd;
    ++n_admit;
  }
  const uint32_t my_rank = (uint32_t)__builtin_popcountll(idle_mask & below) & 15u;
  const uint32_t got_need = (uint32_t)__shfl((int)c_need, (int)my_rank, 64);   // (all lanes take part)
  if (idle && my_rank < n_admit) {
    req = (int32_t)(q_head + my_rank);
    pos = 0;
    held = 0;
    need = got_need;
    nxt = ld_relaxed((const uint32_t*)sv.req_prompt + (size_t)req * sv.max_prompt);
    st_act_u32(sv.req_state + 2 * (size_t)req, 1u);
  }
  q_head += n_admit;
  // ---- (3) the iteration's metadata
  const bool act = mine && req >= 0;
  const bool drained = __ballot(act) == 0ull && q_head >= q_tail;   // nothing running, nothing queued
  const bool wants = act && (pos & ps_mask) == 0u;
  const uint64_t want_mask = __ballot(wants);
  if (wants) {
    const uint32_t idx = n_free - 1u - (uint32_t)__builtin_popcountll(want_mask & below);
    uint32_t pg = lane;   // (never taken: the admission rule keeps promised <= n_free)
    if (idx < n_pages) pg = ld_relaxed((const uint32_t*)sv.free_stack + idx);
    else report(a, DE_BAD_META, 0xFFFFFFFFu, idx);
    const uint32_t blk = pos >> shift;
    if (blk < sv.max_blocks) st_act_u32((uint32_t*)sv.table + (size_t)lane * sv.max_blocks + blk, pg);
    ++held;
  }
  const uint32_t n_popped = (uint32_t)__builtin_popcountll(want_mask);
  n_free -= n_popped;
  promised -= n_popped;
  if (mine) {
    st_act_u32((uint32_t*)sv.slot_req + lane, (uint32_t)req);
    st_act_u32((uint32_t*)sv.slot_pos + lane, act ? pos : 0u);
    st_act_u32((uint32_t*)sv.slot_held + lane, held);
    st_act_u32(tok_io + lane, act ? nxt : 0u);
    st_act_u32(pos_io + lane, act ? pos : 0u);
  }
  if (lane == 0) {
    st_act_u32(sv.scalars + kServeNFree, n_free);
    st_act_u32(sv.scalars + kServePromised, promised);
    st_act_u32(sv.scalars + kServeQHead, q_head);
    st_act_u32(sv.scalars + kServeIterations, ld_relaxed(sv.scalars + kServeIterations) + 1u);
    st_act_u32(sv.scalars + kServeTokens, ld_relaxed(sv.scalars + kServeTokens) + n_produced);
    st_act_u32(sv.scalars + kServeDone, ld_relaxed(sv.scalars + kServeDone) + n_done);
    // nothing running and nothing queued: this iteration is the launch's last (the step number
    // names the decision, so that no stale one is ever taken for it)
    if (drained) st_act_u32(sv.scalars + kServeStop, a.epoch);
  }
}

// D, GRP, NB pin head_dim, query heads per KV head and the batch class at compile time (0 = decide
// at run time): a kernel that carries a single attention and a single linear variant keeps its
// register allocation free of spills, the fully generic kernel does not.
// Batch class -> body instance (NB = 0: decided at run time).
template <int NB, bool MEGA, class Svc = NoJit>
__device__ __forceinline__ uint32_t run_linear(const TaskDesc& t, const StepArgs& a, float* lds, int32_t wait_ev,
                                           uint32_t* s_flag, const Svc& svc = Svc{}, uint32_t next_ti = 0) {
  if (NB == 8) return linear_task_mfma<MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc);   // batch class 5..16: matrix cores
  if (NB == 9) return linear_task<1, MEGA, Svc, true>(t, a, lds, wait_ev, s_flag, svc, next_ti);   // batch 1, large tasks: three buffers
  if (NB != 0) return linear_task<(NB ? NB : 1), MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc, next_ti);
  const uint32_t nb = t.b1 - t.b0;
  if (nb == 1) return linear_task<1, MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc, next_ti);
  if (nb == 2) return linear_task<2, MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc);
  if (nb <= 4) return linear_task<4, MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc);
  return linear_task_mfma<MEGA, Svc>(t, a, lds, wait_ev, s_flag, svc);
}

// Runs one task that is not a linear task.  wait_ev >= 0: the task must first wait for that event
// (persistent kernel); attention tasks do so after requesting their first cache rows.
template <int D, int GRP, int NB>
__device__ __forceinline__ bool run_task(const TaskDesc& t, const StepArgs& a, float* lds,
                                         int32_t wait_ev, uint32_t* s_flag) {
  if (t.kind == TK_ATTN_PARTIAL) {
    if (t.flags & TF_KV_PAGED) {   // paged cache: the same two bodies, rows reached through the page table
      if (D != 0) {
        constexpr uint32_t window = kAttnRounds * (kThreads / 64) * (64 / ((D ? D : 128) / 8));
        if ((GRP ? GRP : 1) <= 4 && !(t.flags & TF_ATTN_BALANCE) && (a.g->max_seq + t.p1 - 1) / t.p1 <= window)
          return body_attn_partial_regs<(D ? D : 128), (GRP ? GRP : 1), true>(t, a, lds, wait_ev, s_flag);
        return body_attn_partial<(D ? D : 128), (GRP ? GRP : 1), true, NB>(t, a, lds, wait_ev, s_flag);
      }
      const uint32_t grp = a.g->n_q / a.g->n_kv;
      if (a.g->head_dim == 128) {
        if (grp == 8) return body_attn_partial<128, 8, true>(t, a, lds, wait_ev, s_flag);
        if (grp == 4) return body_attn_partial<128, 4, true>(t, a, lds, wait_ev, s_flag);
        if (grp == 2) return body_attn_partial<128, 2, true>(t, a, lds, wait_ev, s_flag);
        return body_attn_partial<128, 1, true>(t, a, lds, wait_ev, s_flag);
      }
      if (grp == 8) return body_attn_partial<64, 8, true>(t, a, lds, wait_ev, s_flag);
      if (grp == 4) return body_attn_partial<64, 4, true>(t, a, lds, wait_ev, s_flag);
      if (grp == 2) return body_attn_partial<64, 2, true>(t, a, lds, wait_ev, s_flag);
      return body_attn_partial<64, 1, true>(t, a, lds, wait_ev, s_flag);
    }
    if (D != 0) {
      // chunks that always fit the register-resident body (wavefront-uniform: graph constants)
      constexpr uint32_t window = kAttnRounds * (kThreads / 64) * (64 / ((D ? D : 128) / 8));
      if ((GRP ? GRP : 1) <= 4 && !(t.flags & TF_ATTN_BALANCE) && (a.g->max_seq + t.p1 - 1) / t.p1 <= window)
        return body_attn_partial_regs<(D ? D : 128), (GRP ? GRP : 1)>(t, a, lds, wait_ev, s_flag);
      return body_attn_partial<(D ? D : 128), (GRP ? GRP : 1), false, NB>(t, a, lds, wait_ev, s_flag);
    }
    const uint32_t grp = a.g->n_q / a.g->n_kv;
    if (a.g->head_dim == 128) {
      if (grp == 8) return body_attn_partial<128, 8>(t, a, lds, wait_ev, s_flag);
      if (grp == 4) return body_attn_partial<128, 4>(t, a, lds, wait_ev, s_flag);
      if (grp == 2) return body_attn_partial<128, 2>(t, a, lds, wait_ev, s_flag);
      return body_attn_partial<128, 1>(t, a, lds, wait_ev, s_flag);
    }
    if (grp == 8) return body_attn_partial<64, 8>(t, a, lds, wait_ev, s_flag);
    if (grp == 4) return body_attn_partial<64, 4>(t, a, lds, wait_ev, s_flag);
    if (grp == 2) return body_attn_partial<64, 2>(t, a, lds, wait_ev, s_flag);
    return body_attn_partial<64, 1>(t, a, lds, wait_ev, s_flag);
  }
  if (wait_ev >= 0 && !wait_event(a, wait_ev, s_flag)) return false;
  trace_mark(a, t, 1);
  switch (t.kind) {
    case TK_EMBED: body_embed(t, a); break;
    case TK_RMSNORM: body_rmsnorm(t, lds); break;
    case TK_ROPE: body_rope(t, a); break;
    case TK_ATTN_MERGE: body_attn_merge(t, a); break;
    case TK_ADD: body_add(t); break;
    case TK_SWIGLU: body_swiglu(t); break;
    case TK_ARGMAX: body_argmax(t, a, lds); break;
    case TK_SERVE: body_serve(a); break;
    default: break;   // TK_DUMMY: no computation (normalization, Section 4.1)
  }
  return true;
}

// ------------------------------------------------------------------------------ runtime

// Has event e been activated for this step?  The whole wavefront calls it; the answer is uniform.
// Simple events: one counter, compared with epoch * required by lane 0.  Sharded events (wide,
// all producers ahead-of-time): one counter per producer group (worker index mod 8), each on its
// own 256-byte line; lanes 0..7 read one group's counter each -- a single load instruction -- and
// compare it with epoch * (that group's producers).  An arrival is then ONE atomic add that nobody
// waits for, and 256 producers spread over 8 lines.
__device__ __forceinline__ bool event_reached(const StepArgs& a, int32_t e, int lane) {
  const MPK_CONST EventDesc& ev = *(const MPK_CONST EventDesc*)(a.events + e);
  bool ok = true;
  if (ev.flags & EV_HIER) {
    if (lane < 8) {
      const uint32_t need = a.epoch * ((const MPK_CONST EventDesc*)(a.events + e))->sub_required[lane];
      const uint32_t v = ld_relaxed(a.hier + (size_t)ev.hier_slot * kHierWordsPerEvent + (1 + lane) * kHierStrideWords);
      ok = (int32_t)(v - need) >= 0;
    }
  } else if (lane == 0) {
    ok = (int32_t)(ld_relaxed(a.counters + e) - a.epoch * ev.required) >= 0;
  }
  return __builtin_amdgcn_readfirstlane((int)(__ballot(ok) == ~0ull)) != 0;
}

// The first wavefront polls until event e is activated; *s_flag = 1, or 0 when the step is being
// aborted (watchdog or a peer's failure).  Called by all 64 lanes of the wavefront.
__device__ __forceinline__ void poll_event_wave0(const StepArgs& a, int32_t e, uint32_t* s_flag, int lane) {
  uint32_t ok = 1;
  if (!event_reached(a, e, lane)) {
    const uint64_t t_start = wall_clock64();
    uint32_t it = 0;
    while (!event_reached(a, e, lane)) {
      if ((++it & 255u) == 0) {
        uint32_t dead = 0;
        if (lane == 0) {
          if (ld_relaxed(a.g->err + 1) != 0) dead = 1;
          else if (wall_clock64() - t_start > a.g->timeout_ticks) {
            report(a, DE_TIMEOUT, (uint32_t)e, blockIdx.x);
            __hip_atomic_store(as_global(a.g->err + 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            dead = 1;
          }
        }
        if (__builtin_amdgcn_readfirstlane(dead)) { ok = 0; break; }
      }
    }
  }
  if (lane == 0) *s_flag = ok;
}

// Returns false when the step is being aborted (watchdog or a peer's failure).
__device__ __forceinline__ bool wait_event(const StepArgs& a, int32_t e, uint32_t* s_flag) {
  if (threadIdx.x < 64) poll_event_wave0(a, e, s_flag, (int)threadIdx.x);
  __syncthreads();   // later agent-scope loads cannot move above this barrier
  return __builtin_amdgcn_readfirstlane(*s_flag) != 0;
}

// One lane: add this task's notification to event e (Section 5: "notify the triggering event").
// The arrival that activates an event whose range holds just-in-time tasks hands the event to
// its scheduler's queue.
__device__ __forceinline__ void notify_event(const StepArgs& a, int32_t e) {
  if ((a.flags & kLoseNotifyBit) && blockIdx.x == 0) return;   // MPK_DEBUG_LOSE_NOTIFY: the waiters' watchdog has to end the step
  const MPK_CONST EventDesc& ev = *(const MPK_CONST EventDesc*)(a.events + e);
  const uint32_t flags = ev.flags;
  bool activated = false;
  if (flags & EV_HIER) {
    uint32_t* blk = a.hier + (size_t)ev.hier_slot * kHierWordsPerEvent;
    const uint32_t grp = blockIdx.x & 7u;
    if ((flags & EV_JIT) && a.n_sched) {
      // a scheduler has to be told by the arrival that completes the event: the last arrival of a
      // producer group adds to the top counter, the last of those hands the event over
      uint32_t old = __hip_atomic_fetch_add(as_global(blk + (1 + grp) * kHierStrideWords), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old + 1u == a.epoch * ev.sub_required[grp]) {
        old = __hip_atomic_fetch_add(as_global(blk), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        activated = old + 1u == a.epoch * ev.n_groups;
      }
    } else {
      __hip_atomic_fetch_add(as_global(blk + (1 + grp) * kHierStrideWords), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  } else if ((flags & EV_JIT) && a.n_sched) {
    const uint32_t old = __hip_atomic_fetch_add(as_global(a.counters + e), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    activated = old + 1u == a.epoch * ev.required;
  } else {
    __hip_atomic_fetch_add(as_global(a.counters + e), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (activated && (flags & EV_JIT) && a.n_sched) {
    const uint32_t sc = (uint32_t)e % a.n_sched;
    const uint32_t slot = __hip_atomic_fetch_add(as_global(a.g->evq_tail + sc * 64u), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(as_global(a.g->evq_buf + (size_t)sc * a.g->evq_cap + (slot & (a.g->evq_cap - 1u))),
                       ((uint64_t)(slot + 1u) << 32) | (uint32_t)e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__device__ __forceinline__ void signal_event(const StepArgs& a, const TaskDesc& t, int32_t e) {
  // every wavefront waits until its own agent-scope stores have completed at the coherence point
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  trace_mark(a, t, 6);
  __syncthreads();
  trace_mark(a, t, 7);
  if (threadIdx.x == 0) notify_event(a, e);
}

// Wavefront 0 only: like poll_event_wave0, but also watches the worker's just-in-time queue.
// s_flag[0] = 1 event activated, 0 abort, 2 a just-in-time task (index in s_flag[1]) is queued.
__device__ __forceinline__ void poll_event_or_jit_wave0(const StepArgs& a, int32_t e, uint32_t* s_flag, int lane, uint32_t jit_head) {
  const uint64_t* slot = a.g->wq_buf + (size_t)blockIdx.x * a.g->wq_cap + (jit_head & (a.g->wq_cap - 1u));
  const uint64_t t_start = wall_clock64();
  uint32_t ok, it = 0;
  while (true) {
    if (event_reached(a, e, lane)) { ok = 1; break; }
    uint32_t got = 0, dead = 0;
    if (lane == 0) {
      const uint64_t v = ld_relaxed64(slot);
      if ((uint32_t)(v >> 32) == jit_head + 1u) { s_flag[1] = (uint32_t)v; got = 1; }
      else if ((++it & 127u) == 0) {
        if (ld_relaxed(a.g->err + 1) != 0) dead = 1;
        else if (wall_clock64() - t_start > a.g->timeout_ticks) {
          report(a, DE_TIMEOUT, (uint32_t)e, blockIdx.x);
          __hip_atomic_store(as_global(a.g->err + 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          dead = 1;
        }
      }
    }
    if (__builtin_amdgcn_readfirstlane(got)) { ok = 2; break; }
    if (__builtin_amdgcn_readfirstlane(dead)) { ok = 0; break; }
  }
  if (lane == 0) s_flag[0] = ok;
}

// Wavefront 0 only, after a workgroup barrier: wait for this wavefront's own coherent stores,
// then notify the event.
__device__ __forceinline__ void signal_from_wave0(const StepArgs& a, const TaskDesc& t, int32_t e, int lane) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  trace_mark(a, t, 7);
  if (lane == 0) notify_event(a, e);
}

// The first 192 bytes of the dynamic LDS are control words ([0] = result of the last event wait;
// from word 16: the kernel's arguments); task bodies use the rest.
// The arguments are kept there for the task functions that are real calls: a struct passed by
// value to such a function travels through private memory -- every one of the 512 lanes stores
// and re-loads its own 80-byte copy, 10 MB per call over the chip and a memory round trip before
// the task can start (measured on the MoE shape: 3.9 GB written per step, most of it this).
constexpr uint32_t kLdsArgsAt = 16;
static_assert(kLdsArgsAt * 4 + sizeof(StepArgs) <= kLdsCtrlFloats * 4, "control words too small for the arguments");
// Thread 0 leaves the arguments in LDS; the callers' next barrier publishes them.
__device__ __forceinline__ void publish_args(const StepArgs& a) {
  extern __shared__ __align__(16) float dyn_lds[];
  if (threadIdx.x == 0) *(StepArgs*)(dyn_lds + kLdsArgsAt) = a;
}
__device__ __forceinline__ StepArgs published_args() {
  extern __shared__ __align__(16) float dyn_lds[];
  return uniform_args(*(const StepArgs*)(dyn_lds + kLdsArgsAt));
}
// How a real task function gets the arguments: from LDS (the batch-5..16 kernel, NB = 8, for dense models:
// -1.5 % per step on the batch-8 shape) or by value (the batch-1 kernels, where the LDS form
// measured 0 to +1.3 %, and the mixture-of-experts kernels: +5 % on the MoE shape, also with the
// expert bodies inlined into the task function).
struct ArgsInLds {};
__device__ __forceinline__ StepArgs task_args(const ArgsInLds&) { return published_args(); }
__device__ __forceinline__ StepArgs task_args(const StepArgs& a) { return uniform_args(a); }
template <int NB, bool MOE>
struct TaskArgs {
  using type = std::conditional_t<(NB == 8 && !MOE), ArgsInLds, StepArgs>;
  static __device__ __forceinline__ type make(const StepArgs& a) {
    if constexpr (NB == 8 && !MOE) return ArgsInLds{};
    else return a;
  }
};

// Mixture-of-experts tasks: inlined into run_other_task of the MoE kernels.  (As a real function of
// its own -- so that attention calls would not have to save the many callee-saved registers the
// expert jobs use -- every MoE task paid two nested calls, each with its by-value argument copies
// and register saves: measured 3 to 4 % slower per step on the MoE shape.)
template <bool MEGA>
__device__ __forceinline__ bool run_moe_task(StepArgs a_in, uint32_t task_index, bool skip_wait) {
  const StepArgs a = uniform_args(a_in);
  task_index = uniform_u32(task_index);
  skip_wait = uniform_u32(skip_wait) != 0;
  extern __shared__ __align__(16) float dyn_lds[];
  float* lds = dyn_lds + kLdsCtrlFloats;
  uint32_t* s_flag = (uint32_t*)dyn_lds;
  const TaskDesc t = ld_task(a, task_index);
  if (MEGA) {
    debug_jitter(a, task_index);
    const int32_t wait_ev = (!skip_wait && t.dep_event >= 0 && ((const MPK_CONST EventDesc*)(a.events + t.dep_event))->required != 0) ? t.dep_event : -1;
    trace_mark(a, t, 0);
    if ((a.flags & kTraceBit) && threadIdx.x == 0) as_global(a.g->trace)[(size_t)task_index * kTraceSlots + 5] = blockIdx.x;
    // Cross-task pre-loading (Section 5.3) for the experts' second stage: which experts are active
    // is known since the routing task, long before the first stage has produced this task's
    // inputs.  Such a task (the compiler leaves the routing task's event number + 1 in aux1)
    // waits for that event -- activated before the first stage could start, so this returns at
    // once and only orders the reads of the meta-tensor -- finds its first job and requests that
    // job's first weights, and only then waits for its own event.
    if (wait_ev >= 0 && t.kind == TK_MOE_EXPERT && t.aux1 != nullptr && !(a.flags & kNoPreloadBit)) {
      if (!wait_event(a, (int32_t)(uintptr_t)t.aux1 - 1, s_flag)) return false;
      if (!body_moe_expert(t, a, lds, wait_ev, s_flag)) return false;
      trace_mark(a, t, 3);
      if (t.trig_event >= 0) signal_event(a, t, t.trig_event);
      else __syncthreads();
      trace_mark(a, t, 4);
      return true;
    }
    if (wait_ev >= 0 && !wait_event(a, wait_ev, s_flag)) return false;
    trace_mark(a, t, 1);
  }
  switch (t.kind) {
    case TK_MOE_ROUTE: body_moe_route(t, a, lds); break;
    case TK_MOE_EXPERT: body_moe_expert(t, a, lds); break;
    default: body_moe_combine(t, a); break;
  }
  if (MEGA) {
    trace_mark(a, t, 3);
    if (t.trig_event >= 0) signal_event(a, t, t.trig_event);
    else __syncthreads();
    trace_mark(a, t, 4);
  }
  return true;
}
__device__ __forceinline__ bool is_moe_kind(uint16_t kind) { return kind >= TK_MOE_ROUTE && kind <= TK_MOE_COMBINE; }

// Everything that is not a linear task runs in a function of its own (a real call): its
// thread-index arithmetic and temporaries then get their own register allocation instead of being
// hoisted to the top of the persistent loop, where they would crowd out the weight ring and
// force spills of registers that have loads in flight.
// Returns false when the step is being aborted.
template <int D, int GRP, int NB, bool MEGA, bool MOE>
__device__ __noinline__ bool run_other_task(typename TaskArgs<NB, MOE>::type args, uint32_t task_index, bool skip_wait) {
  const StepArgs a = task_args(args);
  task_index = uniform_u32(task_index);
  skip_wait = uniform_u32(skip_wait) != 0;
  extern __shared__ __align__(16) float dyn_lds[];
  float* lds = dyn_lds + kLdsCtrlFloats;
  uint32_t* s_flag = (uint32_t*)dyn_lds;
  const TaskDesc t = ld_task(a, task_index);
  // (kernels for dense models are built without the mixture-of-experts bodies)
  if (MOE && is_moe_kind(t.kind)) return run_moe_task<MEGA>(a, task_index, skip_wait);
  int32_t wait_ev = -1;
  if (MEGA) {
    debug_jitter(a, task_index);
    wait_ev = (!skip_wait && t.dep_event >= 0 && ((const MPK_CONST EventDesc*)(a.events + t.dep_event))->required != 0) ? t.dep_event : -1;
    trace_mark(a, t, 0);
    if ((a.flags & kTraceBit) && threadIdx.x == 0) as_global(a.g->trace)[(size_t)task_index * kTraceSlots + 5] = blockIdx.x;
  }
  if (!run_task<D, GRP, NB>(t, a, lds, wait_ev, s_flag)) return false;
  if (MEGA) {
    trace_mark(a, t, 3);
    if (t.trig_event >= 0) signal_event(a, t, t.trig_event);
    else __syncthreads();
    trace_mark(a, t, 4);
  }
  return true;
}

__device__ __forceinline__ bool event_active(const StepArgs& a, int32_t e) {
  const MPK_CONST EventDesc& ev = *(const MPK_CONST EventDesc*)(a.events + e);
  if (ev.required == 0) return true;
  if (ev.flags & EV_HIER) {   // (one lane: the eight group counters one after the other, all in flight together)
    const uint32_t* blk = a.hier + (size_t)ev.hier_slot * kHierWordsPerEvent;
    uint32_t v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = ld_relaxed(blk + (1 + k) * kHierStrideWords);
    bool ok = true;
#pragma unroll
    for (int k = 0; k < 8; ++k) ok = ok && (int32_t)(v[k] - a.epoch * ev.sub_required[k]) >= 0;
    return ok;
  }
  return (int32_t)(ld_relaxed(a.counters + e) - a.epoch * ev.required) >= 0;
}


// One scheduler wavefront (Section 5.1): takes activated events from its own queue and hands the
// just-in-time tasks of each event's range to the workers' queues, round-robin from a cursor of
// its own -- local state only, no coordination with other schedulers (Section 6.1).
__device__ __forceinline__ void scheduler_wave(const StepArgs& a, uint32_t sc) {
  const int lane = threadIdx.x & 63;
  const uint32_t W = a.g->n_workers;
  uint32_t head = ld_relaxed(a.g->sched_state + sc * 64u), cursor = ld_relaxed(a.g->sched_state + sc * 64u + 1u);
  uint32_t todo = ld_u32c(a.g->sched_nev + sc);
  // schedulers that hand out the same number of tasks per layer move their cursors in lock-step:
  // start them evenly spread over the workers, or they would all pile onto the same few
  const uint32_t spread = sc * (W / a.n_sched);
  // the start event has no notifications: its owner dispatches it unprompted
  const MPK_CONST EventDesc& sev = *(const MPK_CONST EventDesc*)(a.events + a.g->start_event);
  bool pending_start = (sev.flags & EV_JIT) && a.g->start_event % a.n_sched == sc;
  while (todo > 0 || pending_start) {
    uint32_t e;
    if (pending_start) {
      e = a.g->start_event;
      pending_start = false;
    } else {
      const uint64_t* slot = a.g->evq_buf + (size_t)sc * a.g->evq_cap + (head & (a.g->evq_cap - 1u));
      uint64_t v = ld_relaxed64(slot);
      if ((uint32_t)(v >> 32) != head + 1u) {
        const uint64_t t_start = wall_clock64();
        uint32_t it = 0;
        bool dead = false;
        while ((uint32_t)((v = ld_relaxed64(slot)) >> 32) != head + 1u) {
          if ((++it & 255u) == 0) {
            if (ld_relaxed(a.g->err + 1) != 0) { dead = true; break; }
            if (wall_clock64() - t_start > a.g->timeout_ticks) {
              if (lane == 0) {
                report(a, DE_TIMEOUT, 0x80000000u | sc, blockIdx.x);
                __hip_atomic_store(as_global(a.g->err + 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              }
              dead = true;
              break;
            }
          }
        }
        if (dead) break;
      }
      e = (uint32_t)v;
      ++head;
      --todo;
    }
    const MPK_CONST EventDesc& ev = *(const MPK_CONST EventDesc*)(a.events + e);
    const uint32_t first = ev.first, n = ev.last - ev.first;
    for (uint32_t i = lane; i < n; i += 64) {
      const uint32_t ti = first + i;
      const MPK_CONST TaskDesc& td = *(const MPK_CONST TaskDesc*)(a.tasks + ti);
      if (td.flags & TF_JIT) {
        const uint32_t w = (cursor + spread + i) % W;
        const uint32_t s = __hip_atomic_fetch_add(as_global(a.g->wq_tail + w * 64u), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(as_global(a.g->wq_buf + (size_t)w * a.g->wq_cap + (s & (a.g->wq_cap - 1u))),
                           ((uint64_t)(s + 1u) << 32) | ti, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    cursor += n;
  }
  if (lane == 0) {
    __hip_atomic_store(as_global(a.g->sched_state + sc * 64u), head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(as_global(a.g->sched_state + sc * 64u + 1u), cursor % W, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

constexpr uint32_t kPickExit = 0xFFFFFFFFu, kPickAbort = 0xFFFFFFFEu;

// Worker side of the hybrid launch (Section 5.2): just-in-time tasks first; when none is queued,
// the head of the ahead-of-time queue if its dependent event is activated (or, for a linear task,
// regardless: see linear_wait); exit once the
// ahead-of-time queue is exhausted and the terminal event has been activated.  One lane decides,
// the result goes through LDS.  Returns a task index (bit 31 set: it came from the JIT queue).
__device__ __forceinline__ uint32_t pick_task(const StepArgs& a, uint32_t* ctrl, uint32_t* jit_head, uint32_t* ai, uint32_t q1) {
  if (threadIdx.x == 0) {
    const uint32_t w = blockIdx.x;
    uint32_t pick;
    const uint64_t t_start = wall_clock64();
    uint32_t it = 0;
    while (true) {
      const uint64_t v = ld_relaxed64(a.g->wq_buf + (size_t)w * a.g->wq_cap + (*jit_head & (a.g->wq_cap - 1u)));
      if ((uint32_t)(v >> 32) == *jit_head + 1u) {
        pick = (uint32_t)v | 0x80000000u;
        ++*jit_head;
        break;
      }
      if (*ai < q1) {
        const uint32_t ti = ld_u32c(a.g->aot + *ai);
        const MPK_CONST TaskDesc* td = (const MPK_CONST TaskDesc*)(a.tasks + ti);
        const int32_t dep = td->dep_event;
        // a linear task may start before its event: it requests its weights, then waits for the
        // event itself while serving this worker's just-in-time queue (linear_wait)
        if (dep < 0 || td->kind == TK_LINEAR || event_active(a, dep)) {
          pick = ti;
          ++*ai;
          break;
        }
      } else if (event_active(a, (int32_t)a.g->terminal_event)) {
        pick = kPickExit;
        break;
      }
      if ((++it & 63u) == 0) {
        if (ld_relaxed(a.g->err + 1) != 0) { pick = kPickAbort; break; }
        if (wall_clock64() - t_start > a.g->timeout_ticks) {
          report(a, DE_TIMEOUT, 0x40000000u | (*ai < q1 ? ld_u32c(a.g->aot + *ai) : 0u), blockIdx.x);
          __hip_atomic_store(as_global(a.g->err + 1), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          pick = kPickAbort;
          break;
        }
      }
    }
    ctrl[1] = pick;
    ctrl[2] = *jit_head;
    ctrl[3] = *ai;
  }
  __syncthreads();
  *jit_head = __builtin_amdgcn_readfirstlane(ctrl[2]);
  *ai = __builtin_amdgcn_readfirstlane(ctrl[3]);
  const uint32_t pick = __builtin_amdgcn_readfirstlane(ctrl[1]);
  __syncthreads();   // ctrl may be rewritten only after everybody has read it
  return pick;
}

// Every task ahead-of-time: the worker walks its pre-enqueued list, each task waits for its own
// event.  after_first_step: a task without producers (an embedding task) first waits for the
// previous step's terminal event, i.e. for that step's sampling tasks.  Returns false on abort.
template <int D, int GRP, int NB, bool MOE>
__device__ __forceinline__ bool aot_pass(const StepArgs& a, uint32_t q0, uint32_t q1, float* lds, uint32_t* s_flag,
                                         bool after_first_step) {
  for (uint32_t qi = q0; qi < q1; ++qi) {
    const uint32_t ti = ld_u32c(a.g->aot + qi);
    const TaskDesc t = ld_task(a, ti);
    if (after_first_step && t.dep_event == (int32_t)a.g->start_event) {
      StepArgs prev = a;
      prev.epoch = a.epoch - 1u;
      if (!__builtin_amdgcn_readfirstlane((int)wait_event(prev, (int32_t)a.g->terminal_event, s_flag))) return false;
    }
    if (t.kind == TK_LINEAR) {
      debug_jitter(a, ti);
      const int32_t wait_ev = (t.dep_event >= 0 && ((const MPK_CONST EventDesc*)(a.events + t.dep_event))->required != 0) ? t.dep_event : -1;
      trace_mark(a, t, 0);
      if ((a.flags & kTraceBit) && threadIdx.x == 0) as_global(a.g->trace)[(size_t)t.pad * kTraceSlots + 5] = blockIdx.x;
      // (the next task of this worker: a flagged task pre-loads its first half blocks into LDS pages)
      const uint32_t next_ti = qi + 1 < q1 ? ld_u32c(a.g->aot + qi + 1) : 0u;
      if (!run_linear<NB, true>(t, a, lds, wait_ev, s_flag, NoJit{}, next_ti)) return false;
    } else {
      // the callee's result comes back in a vector register: make it scalar again, or the whole
      // task loop (and every descriptor load in it) turns into per-lane code
      if (!__builtin_amdgcn_readfirstlane((int)run_other_task<D, GRP, NB, true, MOE>(TaskArgs<NB, MOE>::make(a), ti, false))) return false;
    }
  }
  return true;
}

// Serving launches end when the server has drained (Section 5: the kernel runs until the workload
// is done).  The serving task that finds nothing running and nothing queued records its step
// number; steps after that one are not run, but they must still count for the events -- the host
// has advanced the step number for all of them, and events compare counters with step x producers
// -- so every worker adds the notifications of its own tasks, `steps` times each, and leaves.
__device__ __noinline__ void serve_skip_steps(StepArgs a_in, uint32_t q0, uint32_t q1, uint32_t steps) {
  const StepArgs a = uniform_args(a_in);
  q0 = uniform_u32(q0); q1 = uniform_u32(q1); steps = uniform_u32(steps);
  for (uint32_t qi = q0 + threadIdx.x; qi < q1; qi += kThreads) {
    const int32_t e = ((const MPK_CONST TaskDesc*)(a.tasks + ld_u32c(a.g->aot + qi)))->trig_event;
    if (e < 0) continue;
    const MPK_CONST EventDesc& ev = *(const MPK_CONST EventDesc*)(a.events + e);
    uint32_t* cnt = (ev.flags & EV_HIER) ? a.hier + (size_t)ev.hier_slot * kHierWordsPerEvent + (1u + (blockIdx.x & 7u)) * kHierStrideWords
                                         : a.counters + e;
    __hip_atomic_fetch_add(as_global(cnt), steps, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}
// Did an earlier step of this run (steps a.epoch - a.step .. a.epoch - 1) find the server drained?
__device__ __forceinline__ bool serve_drained(const StepArgs& a) {
  const uint32_t stop = __builtin_amdgcn_readfirstlane(ld_relaxed(a.g->serve->scalars + kServeStop));
  return stop - (a.epoch - (uint32_t)a.step) < (uint32_t)a.step;
}

// A launch that is one step of a run: true when an earlier step of the run left the server
// drained -- this step's share of the event counters has then been settled and the kernel leaves.
// (A real call, so that the kernel around it keeps the code it has without it.)
__device__ __noinline__ bool serve_step_gate(StepArgs a_in, uint32_t q0, uint32_t q1) {
  const StepArgs a = uniform_args(a_in);
  if (!(a.flags & kServeBit) || a.step == 0 || !serve_drained(a)) return false;
  serve_skip_steps(a, q0, q1, 1u);
  return true;
}

// Multi-token launch (graphs with the sampling operator, no schedulers): the task list is walked
// n_steps times, the epoch -- hence every counter target -- growing by one each time.  A kernel of
// its own: with the step loop in mpk_mega_kernel the single-step launch measured 2 to 4 % slower.
template <int D, int GRP, int NB, bool MOE>
__global__ void __launch_bounds__(kThreads) mpk_loop_kernel(StepArgs a) {
  extern __shared__ __align__(16) float dyn_lds[];
  float* lds = dyn_lds + kLdsCtrlFloats;
  uint32_t* s_flag = (uint32_t*)dyn_lds;
  const uint32_t w = blockIdx.x;
  const uint32_t q0 = ld_u32c(a.g->aot_off + w), q1 = ld_u32c(a.g->aot_off + w + 1);
  const uint32_t n_steps = a.n_steps;
  for (uint32_t step = 0; step < n_steps; ++step, ++a.epoch) {
    a.step = (uint16_t)step;
    if (step > 0 && (a.flags & kServeBit) && serve_drained(a)) {
      // The previous step's serving task found the server drained; every worker has since run a
      // task downstream of it, so all of them read the same decision here.  The counters move only
      // after that step has ended altogether (its terminal event), or one would pass the target
      // that one of its tasks is still waiting for.
      StepArgs prev = a;
      prev.epoch = a.epoch - 1u;
      if (!wait_event(prev, (int32_t)a.g->terminal_event, s_flag)) return;
      serve_skip_steps(a, q0, q1, n_steps - step);
      return;
    }
    if (NB == 8 && !MOE) {
      __syncthreads();   // (nobody is inside a task function any more)
      publish_args(a);
      __syncthreads();
    }
    if (!aot_pass<D, GRP, NB, MOE>(a, q0, q1, lds, s_flag, step > 0)) return;
  }
}

// PATHS: 0 = the all-ahead-of-time walk and the hybrid launch in one kernel, chosen at run time;
// 1 = ahead-of-time only; 2 = hybrid only.  Which is faster is a matter of register allocation and
// code layout, measured per body: the vector linear body (batch <= 4) runs 0.8 % faster from the
// combined kernel, the matrix-core body spills three times less in a kernel of its own.
// RUN: the instance launched once per step for a run of several steps (vector linear bodies): it
// can find that an earlier step of the run left the server drained.  A kernel of its own, so that
// the single-step kernel stays exactly as it is (1.2 % slower with the check compiled in).
template <int D, int GRP, int NB, bool MOE, int PATHS = 0, bool RUN = false>
__global__ void __launch_bounds__(kThreads) mpk_mega_kernel(StepArgs a) {
  extern __shared__ __align__(16) float dyn_lds[];
  float* lds = dyn_lds + kLdsCtrlFloats;
  uint32_t* s_flag = (uint32_t*)dyn_lds;
  const uint32_t w = blockIdx.x;
  if (NB == 8 && !MOE) {
    publish_args(a);
    __syncthreads();
  }
  if (PATHS != 1 && w >= a.g->n_workers) {
    // scheduler workgroup: 4 scheduler wavefronts (Section 5.1, Table 2), the rest leave
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t sc = (w - a.g->n_workers) * 4u + wave;
    if (wave < 4u && sc < a.n_sched) scheduler_wave(a, sc);
    return;
  }
  const uint32_t q0 = ld_u32c(a.g->aot_off + w), q1 = ld_u32c(a.g->aot_off + w + 1);
  if (PATHS == 1 || (PATHS == 0 && a.n_sched == 0)) {
    // (a run of serving iterations issued as one launch per step: the launches behind the one
    // that found the server drained only settle their share of the event counters)
    if (RUN && __builtin_amdgcn_readfirstlane((int)serve_step_gate(a, q0, q1))) return;
    aot_pass<D, GRP, NB, MOE>(a, q0, q1, lds, s_flag, false);
    return;
  }
  // hybrid launch
  uint32_t jit_head = ld_relaxed(a.g->wq_head + w), ai = q0;
  while (true) {
    const uint32_t pick = pick_task(a, (uint32_t*)dyn_lds, &jit_head, &ai, q1);
    if (pick == kPickExit || pick == kPickAbort) break;
    const uint32_t ti = pick & 0x7FFFFFFFu;
    const TaskDesc t = ld_task(a, ti);
    if (t.kind == TK_LINEAR) {
      debug_jitter(a, ti);
      trace_mark(a, t, 0);
      if ((a.flags & kTraceBit) && threadIdx.x == 0) as_global(a.g->trace)[(size_t)t.pad * kTraceSlots + 5] = blockIdx.x;
      const int32_t wait_ev = (t.dep_event >= 0 && ((const MPK_CONST EventDesc*)(a.events + t.dep_event))->required != 0) ? t.dep_event : -1;
      uint32_t r;
      // started before its event is activated; a just-in-time task that arrives first pre-empts it
      while ((r = run_linear<NB, true>(t, a, lds, wait_ev, s_flag, JitWatch{jit_head})) == kLinPreempted) {
        const uint32_t tj = __builtin_amdgcn_readfirstlane(((uint32_t*)dyn_lds)[1]);
        lds_barrier();   // everybody has read the control word
        ++jit_head;
        // (a just-in-time task may itself be a linear task -- an operator whose tiles read only part
        // of a just-in-time operator's output is labelled just-in-time too, Section 5.2: its event
        // has been activated, so it runs without waiting and without watching the queue)
        const TaskDesc tjd = ld_task(a, tj);
        if (tjd.kind == TK_LINEAR) {
          debug_jitter(a, tj);
          if (run_linear<NB, true>(tjd, a, lds, -1, s_flag) != kLinDone) { r = kLinAbort; break; }
        } else if (!__builtin_amdgcn_readfirstlane((int)run_other_task<D, GRP, NB, true, MOE>(TaskArgs<NB, MOE>::make(a), tj, true))) { r = kLinAbort; break; }
      }
      if (r == kLinAbort) break;
    } else {
      if (!__builtin_amdgcn_readfirstlane((int)run_other_task<D, GRP, NB, true, MOE>(TaskArgs<NB, MOE>::make(a), ti, true))) break;
    }
  }
  if (threadIdx.x == 0) __hip_atomic_store(as_global(a.g->wq_head + w), jit_head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Kernel-per-operator baseline: the same task bodies, one launch per operator, dependencies
// enforced by stream order (what the paper's comparison systems do, Section 6.5).
template <int D, int GRP, int NB, bool MOE>
__global__ void __launch_bounds__(kThreads) mpk_op_kernel(StepArgs a, uint32_t first) {
  extern __shared__ __align__(16) float dyn_lds[];
  float* lds = dyn_lds + kLdsCtrlFloats;
  if (NB == 8 && !MOE) {
    publish_args(a);
    __syncthreads();
  }
  const uint32_t ti = ld_u32c(a.g->op_list + first + blockIdx.x);
  const TaskDesc t = ld_task(a, ti);
  if (t.kind == TK_LINEAR) {
    run_linear<NB, false>(t, a, lds, -1, nullptr);
  } else {
    run_other_task<D, GRP, NB, false, MOE>(TaskArgs<NB, MOE>::make(a), ti, true);
  }
}


// One specialised set of kernels; {0, 0, 0} is the generic fallback.  D, GRP, NB pin head_dim, query
// heads per KV head and the batch class (1: one row, GEMV; 9: one row, three weight buffers; 8: 5..16
// rows, matrix cores); MOE adds the mixture-of-experts task kinds.
struct KernelVariant {
  int d, grp, nb;
  bool moe;
  void (*mega)(StepArgs);     // all tasks ahead-of-time
  void (*op)(StepArgs, uint32_t);
  void (*loop)(StepArgs);
  void (*hybrid)(StepArgs);   // with scheduler workgroups (may be the same kernel as `mega`)
  void (*run_step)(StepArgs); // one step of a run of several, a launch per step (null: use `loop`)
};
// index, head_dim, group, batch class, mixture of experts
#define MPK_VARIANT_LIST(X)                                                                   \
  X(0, 64, 2, 1, false) X(1, 128, 4, 1, false) X(2, 128, 8, 1, false) X(3, 128, 8, 9, false)  \
  X(4, 128, 4, 8, false) X(5, 128, 8, 8, true) X(6, 0, 0, 0, false) X(7, 0, 0, 0, true)
constexpr int kNumVariants = 8;
#define MPK_DECLARE_VARIANT(I, D, G, N, M) const KernelVariant* kernel_variant_##I();
MPK_VARIANT_LIST(MPK_DECLARE_VARIANT)
#undef MPK_DECLARE_VARIANT

}  // namespace mpk
