// Internal structures shared by the host compiler (compiler.cpp) and the HIP runtime
// (runtime.hip).  Nothing here is part of the public ABI.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>

#include "mpk.h"

namespace mpk {

// ---------------------------------------------------------------- device task descriptor
// One fixed-size record per task (paper Section 4.1, "tGraph normalization": after
// normalization a descriptor stores exactly one dependent and one triggering event id, plus
// tensors and configuration).  128 bytes; immutable after compile, so workers may fetch it
// through the scalar cache.
enum TaskKind : uint16_t {
  TK_DUMMY = 0,
  TK_EMBED,
  TK_RMSNORM,
  TK_LINEAR,
  TK_ROPE,
  TK_ATTN_PARTIAL,
  TK_ATTN_MERGE,
  TK_ADD,
  TK_SWIGLU,
  TK_MOE_ROUTE,     // softmax + top-k of every token's router output, builds the meta-tensor
  TK_MOE_EXPERT,    // a share of one expert stage (gate/up or down), sized from the meta-tensor
  TK_MOE_COMBINE,   // weighted sum of a token's expert outputs + residual
  TK_ARGMAX,        // greedy sampling: arg max of one sequence's logits -> next token
  TK_SERVE,         // the task on the start event of a serving graph (paper Section 6.1): retires
                    // finished requests, admits arrivals, updates the paged KV-cache metadata
};

enum TaskFlags : uint16_t {
  TF_PRO_NORM = 1,    // linear: RMSNorm the input row first (gain = w2, eps = f0)
  // (2: unused)
  TF_EPI_RESID = 4,   // linear: out = in2 + W x
  TF_GATEUP = 8,      // linear: out_c = silu(W[c] x) * (W[F + c] x), F = p0
  TF_OUT_LOGITS = 16, // output pointer is the caller's logits buffer of this step
  TF_ROPE_FUSED = 32, // attention: rotate q (and the new k) itself, append k/v itself
  TF_ATTN_MERGE = 64, // attention: the last chunk task of a (sequence, KV head) to finish merges
                      // all chunk partials into the attention output (in2), counter index p2
  TF_JIT = 128,       // launched just-in-time: a scheduler hands it to a worker when its event fires
  TF_QK_NORM = 512,   // rope / attention with fused rope: RMSNorm over head_dim of every q head (gain w)
                      // and k head (gain w2), eps f0, before the rotation
  TF_PAGE_READY = 1024,  // linear (batch 1): this task's first half block per wavefront sits in the LDS page
                         // area, requested there by the worker's previous task
  TF_PAGE_NEXT = 2048,   // linear (batch 1): after its own requests, and before it waits for its event, the
                         // task requests the first half blocks of the worker's NEXT task into the LDS pages
  TF_SPLITK = 256,    // linear (batch > 4): the task owns rows x ONE of `parts` input ranges; it writes
                      // partial sums, and the task of a row block that arrives last (counter p2)
                      // adds the parts in order plus the residual into the real output (aux0).
                      // p1 = weight row length, p3 = parts | part << 8, K = length of the range
  TF_KV_PAGED = 8192, // attention: cache rows are reached through the page table (GraphConst::page_table)
  TF_ATTN_BALANCE = 4096, // attention with fused merge, batch > 1: the batch x C chunk tasks of a KV
                      // head are dealt to the sequences in proportion to their lengths at run time
                      // (a task may work on another sequence than its row; its partial result
                      // still goes to its own slot)
};

struct alignas(16) TaskDesc {
  uint16_t kind, flags;
  int32_t dep_event, trig_event;
  uint32_t b0, b1;   // batch rows [b0, b1)
  uint32_t c0, c1;   // output columns [c0, c1)
  uint32_t K;        // input length (linear / norm), or kind specific
  uint32_t ld_in, ld_out;
  uint32_t p0, p1, p2, p3;  // kind specific
  float f0, f1;             // eps / theta
  const void* w;            // weights (bf16)
  const void* w2;           // gain (bf16)
  const float* in;
  const float* in2;
  float* out;
  void* aux0;               // K cache of the layer
  void* aux1;               // V cache of the layer
  uint64_t pad;
};
static_assert(sizeof(TaskDesc) == 128, "TaskDesc must stay 128 bytes");

struct EventDesc {   // paper Section 4.1 "tGraph linearization" / Fig. 4(f)
  uint32_t required, first, last;
  uint32_t flags;       // bit 0: launches JIT tasks; bit 1: hierarchical arrival (see EV_HIER)
  uint32_t hier_slot;   // index into the hierarchical counter blocks
  uint32_t n_groups;    // worker groups (worker index mod 8) that hold at least one producer
  uint32_t sub_required[8];   // producers per worker group
  uint32_t pad[2];
};
static_assert(sizeof(EventDesc) == 64, "EventDesc is 64 bytes");
constexpr uint32_t EV_JIT = 1, EV_HIER = 2;
// A sharded ("hierarchical") event owns 9 words in use, each on its own 256-byte line: 8 producer-
// group counters (worker index mod 8) that arrivals add to and pollers read all at once (one load
// instruction, a lane per counter), and a top counter used only when a scheduler has to learn which
// arrival was the last.  256 same-address atomics plus 256 pollers on one line cost about 4 us per
// hop on this GPU; sharded, an arrival is one atomic add that nobody waits for.
constexpr uint32_t kHierStrideWords = 64, kHierWordsPerEvent = 17 * kHierStrideWords;
constexpr uint32_t kHierMinRequired = 48;

// ---------------------------------------------------------------- serving state (device)
// What the start-event task of a serving graph keeps in device memory (paper Section 6.1: "the
// KV-cache metadata is stored in device memory for direct access by attention tasks").  One
// record per server; the graph record points to it.  Slots are the batch rows of the graph.
struct ServeDev {
  int32_t* slot_req;         // [batch] request in the slot, -1 = idle
  int32_t* slot_pos;         // [batch] rows cached = position of the token fed this iteration
  int32_t* slot_held;        // [batch] pages the slot's request holds
  int32_t* table;            // [batch][max_blocks] page of (slot, row / page_size); idle slot b: page b
  int32_t* free_stack;       // [kv_pages] free pages, the top is popped first
  uint32_t* scalars;         // kServe* below
  const int32_t* req_prompt; // [max_requests][max_prompt]
  const uint32_t* req_len;   // [max_requests][2]: prompt length, max_new_tokens
  int32_t* req_out;          // [max_requests][max_new]
  uint32_t* req_state;       // [max_requests][2]: 0 pending / 1 running / 2 done, tokens produced
  uint32_t max_blocks, max_prompt, max_new, max_requests;
  int32_t eos;
  uint32_t page_shift;
};
enum : uint32_t { kServeNFree = 0, kServePromised = 1, kServeQHead = 2, kServeQTail = 3, kServeIterations = 4,
                  kServeTokens = 5, kServeDone = 6, kServeStop = 7, kServeScalars = 8 };

// ---------------------------------------------------------------- host-side graph
struct HostOp {
  uint32_t kind;     // MPK_OP_*
  int32_t layer;
  std::string name;
  uint32_t rows, cols, unit;   // output tensor [rows][cols]; columns tile in multiples of unit
  uint32_t tb, tc;
  uint32_t task_base;          // canonical id of tile 0
  uint32_t jit;
  // tensors
  int out_tensor;
  int in_tensor, in2_tensor;   // -1 if none (dependency analysis reads these)
  int body_in_tensor = -1;     // tensor the body actually loads when it differs from in_tensor
  int side_out_tensor = -1;    // second output written by the body (merged attention output)
  int in3_tensor = -1;         // third tensor the dependency analysis reads (combine: meta-tensor)
  int body_in2_tensor = -1;    // tensor the body loads as second input when it differs from in2_tensor
  uint32_t in_kparts = 0, in2_kparts = 0;   // the input is a split-K operator's partial tensor with this many parts
  // mixture-of-experts operators: the tensors the body really touches (the dependency analysis
  // sees an expert stage's output as one element per task, see build_ops)
  int data_in = -1, data_in2 = -1, data_out = -1, data_aux = -1;
  uint32_t align_unit = 0;     // linear: no tile straddles a multiple of this (head_dim) when non-zero
  uint32_t seg_tiles = 0;      // ... by a two-level split: segments of align_unit columns, this many tiles each
  std::vector<uint32_t> col_begin;   // explicit column tiles (tc + 1 starts, in units) when not empty: tiles
                                     // sized by the speed of the worker that runs them
  // parameters
  uint32_t K;
  uint16_t flags;
  const void *w, *w2;
  float f0, f1;
  uint32_t p0, p1, p2, p3;
};

struct HostTask {   // linearized order
  uint32_t op;      // MPK_TASK_DUMMY_OP for dummies
  uint32_t tile;
  int32_t dep_event, trig_event;
  int32_t worker;
  uint32_t jit;
};

struct HostTensor {
  uint32_t rows, cols;
  size_t offset;   // float offset into the activation arena; SIZE_MAX = external (logits)
};

struct HostGraph {
  mpk_model_config cfg{};
  mpk_compile_options opt{};
  std::vector<HostOp> ops;
  std::vector<HostTensor> tensors;
  std::vector<HostTask> tasks;
  std::vector<EventDesc> events;
  std::vector<uint32_t> aot_off, aot;
  std::vector<TaskDesc> descs;   // parallel to tasks; activation pointers hold arena offsets
                                 // until the runtime relocates them
  uint32_t n_real = 0, start_event = 0, terminal_event = 0;
  size_t arena_floats = 0;
  uint32_t lds_bytes = 0;
  uint32_t n_group_counters = 0;   // arrival counters: per (layer, sequence, KV head), then per split-K row block
  uint32_t n_group_counters_attn = 0, n_splitk_counters = 0;
  uint32_t n_hier_events = 0;
  uint32_t lin_rows_max = 0;       // largest weight-row count of one linear task (gate/up pairs twice)
  uint32_t lin_res_rows_max = 0;   // largest column count of a linear task with a residual epilogue
  uint32_t lin_page_off = 0;       // float offset (in the task area of the LDS) of the pre-load pages, 0 = none
  std::vector<size_t> moe_meta_offset;   // per MoE layer: float offset of its meta-tensor in the arena
  std::vector<double> inv_freq;    // RoPE frequencies theta^(-2i/d), i < d/2
  mpk_stats stats{};
};

void set_error(const char* fmt, ...);

// compiler.cpp
mpk_status build_model_graph(const mpk_model_config& cfg, const mpk_weight_ptrs* w,
                             const mpk_kv_ptrs* kv, const mpk_compile_options& opt, HostGraph& g);
mpk_status build_dag_graph(uint32_t n_tasks, const uint32_t* pairs, size_t n_pairs,
                           const mpk_compile_options& opt, HostGraph& g);

// Meta-tensor of one mixture-of-experts layer (Section 6.4), 32-bit words, E experts, P = batch x
// top_k (token, rank) pairs; pair p = token * top_k + rank, ranks in ascending expert index:
//   [0] number of active experts   [1] largest token count of one expert
//   [2 .. 2+E)        active experts, ascending
//   [2+E .. 2+2E)     tokens per expert
//   [2+2E .. 2+3E)    first entry of each expert in the pair list
//   [2+3E .. +P)      pair list, sorted by (expert, token)
//   [2+3E+P .. +P)    combine weight of pair p (float)
//   [2+3E+2P .. +P)   expert of pair p
inline uint32_t moe_meta_words(uint32_t E, uint32_t P) { return 2 + 3 * E + 3 * P; }

// Section 6.4, the run-time refinement: which of the active experts' 16-row weight tiles -- laid
// end to end in ascending expert order, n_active x tiles_per_expert of them -- expert task `task`
// of `n_tasks` works on: [*first, *last).  A task whose share crosses from one expert into the
// next works it off in two jobs, and the change-over (epilogue, staging, the first weights with
// nothing requested ahead) costs about as much as kMoeSwitchTiles tiles, so the shares are equal
// in COST: every expert counts as its tiles plus a gap of kMoeSwitchTiles, the tasks divide that
// axis evenly, and position x on it maps back to tile min(x mod period, tiles) of expert
// x / period.  A pure function of its arguments (host and device compute the same split); the
// shares are disjoint, in order, and cover every tile.
constexpr uint32_t kMoeSwitchTiles = 8;   // (4: +1.5 % per step on the mixture-of-experts shape; 7 and 10: the same as 8)
#if defined(__HIPCC__)
#define MPK_HOST_DEVICE __host__ __device__
#else
#define MPK_HOST_DEVICE
#endif
MPK_HOST_DEVICE inline void moe_task_share(uint32_t n_active, uint32_t tiles_per_expert, uint32_t n_tasks, uint32_t task,
                                           uint32_t* first, uint32_t* last) {
  const uint64_t period = (uint64_t)tiles_per_expert + kMoeSwitchTiles, cost = (uint64_t)n_active * period;
  const uint64_t x0 = cost * task / n_tasks, x1 = cost * ((uint64_t)task + 1u) / n_tasks;
  const uint64_t r0 = x0 % period, r1 = x1 % period;
  *first = (uint32_t)(x0 / period) * tiles_per_expert + (uint32_t)(r0 < tiles_per_expert ? r0 : tiles_per_expert);
  *last = (uint32_t)(x1 / period) * tiles_per_expert + (uint32_t)(r1 < tiles_per_expert ? r1 : tiles_per_expert);
}
constexpr uint32_t kMoeMaxExperts = 512, kMoeMaxPairs = 256, kMoeMaxTopK = 16;

// Matrix-core jobs (batch 5..16 and expert jobs) stage the input in LDS as fp32, a chunk of this
// many inputs at a time; one definition for the host's LDS requirement and the kernels' layout.
constexpr uint32_t mfma_kchunk(uint32_t nb) { return nb <= 8u ? 4096u : 2048u; }
constexpr uint32_t kMfmaXPad = 32;   // floats between staged rows beyond the chunk (bank spread)
// LDS floats of a job with nb staged rows: nb rows x (chunk + pad) f32 (reused for the partial
// tiles [8 wavefronts][4][16][16] f32 at the end), then the chunk's RMSNorm gains as bf16.
constexpr uint32_t mfma_x_floats(uint32_t nb) {
  const uint32_t x = nb * (mfma_kchunk(nb) + kMfmaXPad);
  return (x > 8u * 4u * 256u ? x : 8u * 4u * 256u) + mfma_kchunk(nb) / 2u;
}
// ... of the expert jobs of a graph with this batch size: an expert holds between 1 and min(batch,
// 16) token rows.
constexpr uint32_t moe_x_floats(uint32_t batch) {
  const uint32_t t8 = mfma_x_floats(batch < 8u ? batch : 8u);
  const uint32_t t16 = batch > 8u ? mfma_x_floats(batch < 16u ? batch : 16u) : 0u;
  return t8 > t16 ? t8 : t16;
}

// LDS layout constants shared with the kernels
constexpr uint32_t kThreads = 512;        // worker workgroup size (8 wavefronts, two per SIMD)
constexpr uint32_t kLdsReduceFloats = 1024;  // scratch for cross-wave reductions
constexpr uint32_t kLdsCtrlFloats = 48;      // control words ahead of the task area (event-wait result, the kernel's arguments)
constexpr uint32_t kMinLdsBytes = 84 * 1024; // > half of 160 KB: at most one worker per CU
// Pre-load pages in LDS (paper Section 5.3: shared-memory pages hold data pre-loaded for a task that
// has not started): one page of 16 KB per wavefront = one half block of the vector linear body.
constexpr uint32_t kLinPageFloats = 4096, kLinPagesFloats = 8 * kLinPageFloats;
constexpr uint32_t kLinPageUnits = 16;   // weight rows one set of pages holds: 8 wavefronts x 2 rows

}  // namespace mpk
