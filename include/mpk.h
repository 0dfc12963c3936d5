/*
 * mpk.h -- C ABI of the MI355X task-graph mega-kernel decoder.
 *
 * One LLM decode step (embedding; per layer RMSNorm, QKV projection, RoPE, decode attention over
 * the KV cache, O projection, residual, RMSNorm, SwiGLU MLP, residual; final RMSNorm; LM head) is
 * compiled on the host into a CU-level task graph ("tGraph", paper Section 3) and executed by one
 * persistent HIP kernel (paper Section 5).
 *
 * Conventions used by every entry point
 *   - "host" / "device" on a pointer says where the memory must live.  Device pointers are plain
 *     HIP device allocations of the GPU that was current when mpk_compile was called.
 *   - The library BORROWS every pointer handed to mpk_compile for the lifetime of the graph and
 *     never frees it.  The library OWNS the graph object and everything it allocates (task and
 *     event tables, queues, event counters, fp32 activation buffers); mpk_graph_destroy frees it.
 *   - No function throws or aborts.  Failures return a status code; mpk_last_error() gives a
 *     thread-local message that stays valid until the next call on the same thread.
 *   - `stream` arguments are a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef MPK_H
#define MPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MPK_OK = 0,
  MPK_ERR_INVALID_ARG = 1, /* null pointer, zero size, bad struct_size, misaligned pointer    */
  MPK_ERR_UNSUPPORTED = 2, /* a shape the task bodies cannot tile (see mpk_compile)           */
  MPK_ERR_OOM = 3,         /* host or device allocation failed                                */
  MPK_ERR_RESIDENCY = 4,   /* the persistent kernel's workgroups cannot all be co-resident    */
  MPK_ERR_HIP = 5,         /* a HIP call failed; message holds the HIP error string           */
  MPK_ERR_TIMEOUT = 6,     /* the in-kernel watchdog fired (an event never activated)         */
  MPK_ERR_INTERNAL = 7,    /* compiler invariant violated                                     */
  MPK_ERR_DEVICE = 8       /* the kernel reported an error (e.g. position >= max_seq, a page
                              table entry outside the pool)                                   */
} mpk_status;

/* ----------------------------------------------------------------------------------------------
 * Model description.  Sizes are element counts.  All weights are bf16, row-major [out][in];
 * the fused QKV matrix stacks the query rows, then the key rows, then the value rows; the fused
 * gate/up matrix stacks the gate rows [0, ffn) then the up rows [ffn, 2 ffn).  Activations are
 * fp32 inside the library.  The paper fixes none of these layouts (it names the operators only,
 * Section 4 Fig. 4 and Section 6.5); they are this library's contract.
 * -------------------------------------------------------------------------------------------- */
typedef struct mpk_model_config {
  uint32_t struct_size; /* = sizeof(mpk_model_config) */
  uint32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps, rope_theta;
  uint32_t batch;   /* the graph is specialised for this batch size (Section 6.1, "supporting
                       runtime dynamism": one tGraph per batch size)                              */
  uint32_t max_seq; /* KV-cache capacity per sequence, in positions                              */
  uint32_t n_experts, top_k, expert_ffn; /* 0 = dense MLP                                        */
  uint32_t flags;                        /* MPK_MODEL_* bits                                     */
} mpk_model_config;

/* mpk_model_config.flags */
#define MPK_MODEL_QK_NORM 1u /* RMSNorm over head_dim of every q and k head, with gains q_norm /
                                k_norm and rms_eps, before RoPE (the Qwen3 family)              */

typedef struct mpk_layer_weights {
  const void *attn_norm; /* device bf16 [hidden]                                   */
  const void *wqkv;      /* device bf16 [(n_q + 2 n_kv) head_dim][hidden]          */
  const void *wo;        /* device bf16 [hidden][n_q head_dim]                     */
  const void *mlp_norm;  /* device bf16 [hidden]                                   */
  const void *wgu;       /* device bf16 [2 ffn][hidden]           (dense)          */
  const void *wd;        /* device bf16 [hidden][ffn]             (dense)          */
  const void *router;    /* device bf16 [n_experts][hidden]       (MoE)            */
  const void *expert_wgu; /* device bf16 [n_experts][2 expert_ffn][hidden] (MoE)   */
  const void *expert_wd;  /* device bf16 [n_experts][hidden][expert_ffn]   (MoE)   */
  const void *q_norm;    /* device bf16 [head_dim]   (MPK_MODEL_QK_NORM)            */
  const void *k_norm;    /* device bf16 [head_dim]   (MPK_MODEL_QK_NORM)            */
} mpk_layer_weights;

typedef struct mpk_weight_ptrs {
  const void *embed;      /* device bf16 [vocab][hidden]                            */
  const void *final_norm; /* device bf16 [hidden]                                   */
  const void *lm_head;    /* device bf16 [vocab][hidden] (not tied to `embed`)      */
  const mpk_layer_weights *layers; /* HOST array [n_layers] of device pointers      */
} mpk_weight_ptrs;

/* KV cache: bf16, layout [n_layers][batch][n_kv_heads][max_seq][head_dim], one allocation each.
 * A decode step WRITES row positions[b] of every (layer, b, kv head) and READS rows
 * 0..positions[b] (the freshly written row included, as rounded to bf16). */
typedef struct mpk_kv_ptrs {
  void *k; /* device */
  void *v; /* device */
} mpk_kv_ptrs;

/* Operator fusions applied when the operator list is built (before decomposition). */
#define MPK_FUSE_NORM 1u   /* RMSNorm folded into the linear operator that consumes it          */
#define MPK_FUSE_RESID 2u  /* residual add folded into the producing linear operator's epilogue */
#define MPK_FUSE_SWIGLU 4u /* gate/up projection emits silu(gate)*up directly                   */
#define MPK_FUSE_MERGE 8u  /* split-KV merge done by the last attention chunk task to finish    */
#define MPK_FUSE_ROPE 16u  /* RoPE + KV append folded into the attention tasks                  */

#define MPK_DEBUG_TRACE 1u  /* record per-task timestamps inside the persistent kernel          */
#define MPK_DEBUG_POISON 2u /* before every launch, fill every buffer the graph owns for data that
                               crosses tasks (activations, split-KV partials, partial sums,
                               meta-tensors) with NaN, and leave NaN patterns in the compute
                               units' local data share: a task that reads what this step has not
                               produced yet, what an earlier step left behind, or a word of its
                               staging area that it has not written, shows in the logits (the
                               paper's runtime has no such mode; Section 5 only states that
                               events order producers before consumers)                          */
#define MPK_DEBUG_JITTER 4u /* every task of the persistent kernel starts after a pseudo-random
                               delay of 0 .. 20 us (a hash of task and step): the relative timing
                               of producers and consumers differs in every step, so a missing
                               wait or an early notification becomes a wrong result.  All waits
                               stay bounded; nothing hangs or faults on purpose                  */

#define MPK_LAUNCH_MEGA 0u   /* one persistent kernel per decode step (Section 5)               */
#define MPK_LAUNCH_PER_OP 1u /* same task bodies, one kernel launch per operator (baseline)     */

#define MPK_DEBUG_LOSE_NOTIFY 8u /* the FIRST persistent-kernel launch of the graph loses worker
                               0's notifications: the events they belong to never activate, every
                               wait that depends on them ends at its watchdog limit
                               (spin_timeout_ms), all workgroups exit, and mpk_graph_status reports
                               MPK_ERR_TIMEOUT.  For testing that path and mpk_graph_reset        */

typedef struct mpk_compile_options {
  uint32_t struct_size;     /* = sizeof(mpk_compile_options)                                    */
  uint32_t n_workers;       /* worker workgroups, one per CU (Section 5); 0 = all CUs minus the
                               scheduler CUs (host_only: 256 - n_sched_wgs)                     */
  uint32_t n_sched_wgs;     /* scheduler workgroups, 4 scheduler wavefronts each (Section 5,
                               Table 2 uses 4 SMs x 4 warps); 0 = no schedulers: every operator
                               is launched ahead of time                                        */
  uint32_t fusion;          /* MPK_FUSE_* bits                                                  */
  uint32_t transitive_reduction; /* 1 = drop producer->consumer pairs implied by other pairs
                               before event fusion (not in the paper; removes fork/join dummies
                               caused by residual connections)                                  */
  uint32_t attn_chunks;     /* KV splits per (sequence, KV head); 0 = auto                      */
  uint32_t tiles_linear;    /* tasks per linear operator (Section 4.1: "proportional to the
                               number of SMs", user-settable); 0 = n_workers                    */
  uint32_t tiles_lm_head;   /* tasks for the LM head; 0 = n_workers                             */
  uint32_t tiles_pointwise; /* column tiles per batch row of add / swiglu operators; 0 = 1     */
  uint32_t launch_mode;     /* MPK_LAUNCH_*                                                     */
  uint32_t force_aot;       /* 1 = label every operator ahead-of-time even with schedulers      */
  uint32_t no_preload;      /* 1 = switch cross-task pre-loading off (Section 5.3; the ablation
                               of Section 6.5, Fig. 10): no task requests weights or cache rows
                               before its dependent event is activated.  0 = pre-loading on     */
  uint32_t host_only;       /* 1 = build the task graph on the host only: no device is touched,
                               weight/KV pointers may be NULL; mpk_decode_step is refused       */
  uint32_t spin_timeout_ms; /* in-kernel watchdog for every wait; 0 = 2000 ms                   */
  uint32_t debug_flags;     /* MPK_DEBUG_* bits                                                 */
  uint32_t tiles_moe;       /* expert tasks per expert stage of a mixture-of-experts layer
                               (Section 6.4: expert tasks are fixed at compile time and split
                               the active experts' rows evenly at run time); 0 = n_workers      */
  uint32_t greedy_loop;     /* 1 = append a greedy-sampling operator (arg max of the logits,
                               lowest index on ties; tiles_sampling tasks per sequence) so that several
                               tokens can be decoded in ONE launch (mpk_decode_steps): the
                               kernel runs until its workload is done (Section 5).  Such a
                               graph is run with mpk_decode_steps only.  How n steps are
                               issued is the library's choice: one launch of the persistent
                               kernel, or -- for the model shapes the library has specialised
                               kernels for, whose linear bodies run 1 to 3.5 % slower inside
                               the step loop and whose paged attention needs slower loads
                               inside a launch of several steps -- n launches of the
                               single-step kernel back to back, with no host synchronisation
                               between them; 2 = always the one launch                          */
  uint32_t kv_batch;        /* number of sequences the KV cache is laid out for (the `batch`
                               extent of mpk_kv_ptrs' layout); 0 = cfg.batch.  Lets a graph for
                               fewer sequences run on the first cfg.batch slots of a larger
                               cache (mpk_compile_set)                                          */
  uint32_t worker_weight_permille[8]; /* relative streaming speed of the workers with index mod 8
                               == k (the XCD a workgroup lands on), in thousandths; all 0 = equal.
                               When they differ, the column tiles of a linear operator are sized in
                               proportion to the speed of the worker that runs each (Section 4.1
                               leaves the partition to the compiler: "the partitioning strategy
                               ... minimizes device memory loading"; an operator ends with its
                               slowest task).  Batch <= 4, operators with one tile per row block
                               and at least 64 weight rows per tile, all tasks ahead-of-time; the
                               exported graph lists the boundaries                              */
  uint32_t no_lds_pages;    /* 1 = no pre-load pages in LDS.  By default, at batch 1 without
                               scheduler workgroups, a worker that has a long wait ahead (the O
                               projection behind the attention tasks) requests the first 16 KB
                               per wavefront of the task AFTER that one into LDS pages while it
                               waits (Section 5.3: pre-loading into shared-memory pages across
                               tasks); that task's tile is made correspondingly larger than the
                               tiles of workers that could not pre-load (they ran attention)    */
  uint32_t xcd_balance;     /* 1 = measure those speeds on this GPU at compile time (a streaming
                               kernel over the LM-head weights, about a millisecond) when
                               worker_weight_permille is all 0.  Not with host_only              */
  uint32_t no_attn_balance; /* 1 = every sequence keeps its own attn_chunks attention tasks.  By
                               default (batch > 1, merge fused into the attention tasks) the
                               batch x attn_chunks tasks of a KV head are dealt to the sequences
                               in proportion to their current lengths when the step runs, one at
                               least each: with a ragged batch an attention operator otherwise
                               ends with the longest sequence's chunks (the run-time imbalance
                               Section 5.2 meets with just-in-time hand-out; here the split is
                               a pure function of the positions, so results stay reproducible)   */
  uint32_t kv_page_size;    /* 0 = contiguous KV cache.  Otherwise the cache is PAGED (Section 6.1,
                               paged attention): rows per page, a power of two >= 8 that divides
                               max_seq.  mpk_kv_ptrs then points to pools laid out
                               [n_layers][kv_pages][n_kv_heads][kv_page_size][head_dim], and row r
                               of sequence b lives in page page_table[b][r / kv_page_size] (the
                               same page number in every layer).  The table is device memory: the
                               serving task's (serving = 1) or the caller's
                               (mpk_graph_set_page_table).  Needs MPK_FUSE_ROPE; kv_batch must
                               be 0                                                             */
  uint32_t kv_pages;        /* pages per layer in the pools (with kv_page_size)                 */
  uint32_t serving;         /* 1 = the graph starts with the serving task (Section 6.1: ONE task
                               on the start event removes completed requests, admits arrivals and
                               updates the KV-cache metadata in device memory).  Needs
                               greedy_loop = 1, kv_page_size > 0, no scheduler workgroups.  Such
                               a graph is run through its server only: mpk_serve_run             */
  uint32_t tiles_sampling;  /* tasks per sequence of the sampling operator (greedy_loop): each scans
                               a share of the logits as soon as the LM-head tasks that produce it
                               are done, the one to finish last picks the token.  0 = one per 8192
                               logits (at most 32)                                              */
} mpk_compile_options;

typedef struct mpk_graph mpk_graph;

/* Compile one decode step for `cfg` into a task graph (Section 4.1: operator decomposition,
 * dependency analysis, event fusion, normalization, linearization; Section 5.2: launch-mode
 * labelling and ahead-of-time pre-enqueue) and upload it.
 *   cfg, weights, kv : host structs (see above); weights/kv may be NULL only with host_only.
 *   opts             : host, may be NULL (all defaults).
 *   out              : host, receives the graph handle (NULL on failure).
 * Errors: INVALID_ARG (null/zero/misaligned: every weight pointer must be 16-byte aligned),
 * UNSUPPORTED (head_dim not 64 or 128; hidden, ffn or n_q*head_dim not a multiple of 8;
 * n_q not a multiple of n_kv; batch > 16; mixture-of-experts layers with more than 512 experts,
 * top_k > 16, batch x top_k > 256, expert_ffn not a multiple of 8 or hidden not of 16),
 * RESIDENCY, OOM, HIP. */
mpk_status mpk_compile(const mpk_model_config *cfg, const mpk_weight_ptrs *weights,
                       const mpk_kv_ptrs *kv, const mpk_compile_options *opts, mpk_graph **out);

/* Compile an explicit task DAG (diagnostics and tests of the graph passes of Section 4.1 on
 * arbitrary graphs): tasks 0..n_tasks-1, `pairs` = host array of n_pairs (producer, consumer)
 * u32 pairs.  The result is a host-only graph: event fusion, normalization, linearization and
 * round-robin pre-enqueue are applied exactly as in mpk_compile; it can be exported, not run. */
mpk_status mpk_compile_dag(uint32_t n_tasks, const uint32_t *pairs, size_t n_pairs,
                           const mpk_compile_options *opts, mpk_graph **out);

/* Run one decode step (Section 6.1: calling the compiled object issues a single mega-kernel
 * launch).  Asynchronous on `stream`; no host synchronisation, no allocation.
 *   token_ids  : device int32 [batch]
 *   positions  : device int32 [batch]; positions[b] = number of rows already cached for b
 *   logits_out : device fp32 [batch][vocab], written by the LM-head tasks
 * A position >= max_seq or a token outside [0, vocab) is detected in the kernel and reported by
 * mpk_graph_status.  Steps of one graph must not overlap (same stream, or externally ordered).
 * The step number is a launch argument that events are compared against: a persistent-kernel
 * launch must not be captured into a HIP graph and replayed (the replays would carry the captured
 * step number); MPK_LAUNCH_PER_OP launches use no events and may be captured. */
mpk_status mpk_decode_step(mpk_graph *g, const int32_t *token_ids, const int32_t *positions,
                           float *logits_out, void *stream);

/* Decode n_steps tokens greedily in one call, with no host round trip between tokens (Section 5:
 * the kernel keeps running until the workload completes): one launch of the persistent kernel, or
 * a launch per step issued back to back (see greedy_loop).  Only for graphs compiled with
 * greedy_loop and without scheduler workgroups; with MPK_LAUNCH_PER_OP the host
 * issues the operator kernels of every step instead.
 *   token_ids  : device int32 [batch], IN: the tokens to feed first; OUT: the last tokens sampled
 *   positions  : device int32 [batch], IN: rows already cached; OUT: advanced by n_steps
 *   tokens_out : device int32 [n_steps][batch] or NULL: the token sampled at every step
 *   logits_out : device fp32 [batch][vocab]: logits of the LAST step
 *   logits_all : device fp32 [n_steps][batch][vocab] or NULL: a copy of every step's logits
 * Step s reads and appends K/V rows at positions[b] + s; every position must stay below max_seq.
 * Asynchronous on `stream`; errors as mpk_decode_step. */
mpk_status mpk_decode_steps(mpk_graph *g, uint32_t n_steps, int32_t *token_ids, int32_t *positions,
                            int32_t *tokens_out, float *logits_out, float *logits_all, void *stream);

/* mpk_decode_step for callers that must not allocate device memory and want the library to hold
 * none for them per graph either (code under HIP graph capture of the per-operator launches,
 * tight serving loops, harnesses that forbid hipMalloc): the step's scratch memory -- activations,
 * split-KV partials, partial sums, meta-tensors, event and arrival counters -- lives in ONE array
 * of MPK_STATIC_SCRATCH_BYTES that is part of the library image (each GPU the library runs on
 * holds its copy until the process ends), not in the buffers mpk_compile allocated for the graph.
 * The call itself allocates nothing and frees nothing.
 *   Arguments, outputs and errors as mpk_decode_step.  Additionally UNSUPPORTED when the graph
 *   needs more scratch than the array holds (mpk_static_scratch_need tells), when it was compiled
 *   with scheduler workgroups, greedy_loop or MPK_DEBUG_TRACE, or host_only.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU race, also
 * calls of different graphs.  The array keeps the previous call's contents; the call clears the
 * counters it needs at zero itself (a small kernel on `stream`, no memset node) and every step
 * counts as the graph's first, so steps through this entry point and through mpk_decode_step may
 * be mixed freely on one graph. */
#define MPK_STATIC_SCRATCH_BYTES (32u << 20)
mpk_status mpk_decode_step_static(mpk_graph *g, const int32_t *token_ids, const int32_t *positions,
                                  float *logits_out, void *stream);
/* Bytes of scratch a step of this graph needs (what mpk_decode_step_static places in the array). */
size_t mpk_static_scratch_need(const mpk_graph *g);

/* After the stream has been synchronised by the caller: translate the device error word.
 * MPK_OK, MPK_ERR_TIMEOUT (watchdog; the graph must be reset) or MPK_ERR_DEVICE. */
mpk_status mpk_graph_status(mpk_graph *g);

/* Clear event counters, queues and the error word (after a TIMEOUT).  Synchronises the device. */
mpk_status mpk_graph_reset(mpk_graph *g);

typedef struct mpk_stats {
  uint32_t struct_size;
  uint32_t n_ops;          /* operators after fusion flags                                     */
  uint32_t n_tasks;        /* tasks in the final graph, dummy tasks included                    */
  uint32_t n_dummy_tasks;  /* inserted by normalization                                         */
  uint32_t n_events;       /* events in the final graph (start and terminal events included)   */
  uint32_t n_events_fused; /* events after the two fusion passes, before normalization          */
  uint64_t n_pair_deps;    /* producer-consumer task pairs = events before fusion               */
  uint64_t n_pairs_removed;/* pairs dropped by transitive reduction                             */
  uint32_t n_jit_tasks, n_aot_tasks;
  uint32_t n_workers, n_sched_wgs;
  uint32_t lds_bytes;      /* dynamic LDS per workgroup                                         */
  uint32_t task_desc_bytes;/* size of one device task descriptor                                */
  uint64_t successor_bytes_unlinearized; /* 4 B per (event, launched task) entry                */
  uint64_t successor_bytes_linearized;   /* 8 B per event (first, last)                         */
  uint64_t weight_bytes;   /* bf16 weight bytes one step streams (embedding rows included)      */
  uint64_t kv_row_bytes;   /* K+V bytes read per cached position, summed over layers & kv heads */
  uint64_t act_bytes;      /* fp32 activation buffers owned by the graph                        */
  uint64_t expert_bytes;   /* mixture-of-experts: bf16 bytes of ONE expert of one layer (gate, up
                              and down matrices); weight_bytes then excludes the experts: a step
                              streams weight_bytes + expert_bytes x (distinct experts selected,
                              summed over layers, see mpk_graph_moe_active)                    */
} mpk_stats;

mpk_status mpk_graph_stats(const mpk_graph *g, mpk_stats *out);

/* Export the compiled graph (host memory, little-endian, see the mpk_export_* structs).
 * Layout: header | ops[n_ops] | tasks[n_tasks] (linearized order) | events[n_events] |
 * u32 aot_offsets[n_workers + 1] | u32 aot_tasks[aot_offsets[n_workers]] | u32 n_explicit |
 * n_explicit x { u32 op, u32 n (= that operator's tc + 1), u32 column_begin[n] }: the operators
 * whose column tiles are not the even split (worker_weight_permille), with their boundaries.
 * Call with buf == NULL to get the size in *need.  INVALID_ARG if cap is too small. */
#define MPK_EXPORT_MAGIC 0x4B504D54u /* "TMPK" */
#define MPK_NO_EVENT (-1)
#define MPK_TASK_DUMMY_OP 0xFFFFFFFFu

typedef struct mpk_export_header {
  uint32_t magic, version, n_ops, n_tasks, n_events, n_workers, n_sched_wgs, start_event;
  uint32_t terminal_event, n_real_tasks, fusion, reserved;
} mpk_export_header;

typedef struct mpk_export_op {
  uint32_t kind;  /* MPK_OP_*                                          */
  int32_t layer;  /* -1 for embedding / final norm / LM head           */
  uint32_t tb, tc; /* partition degree along batch rows and columns    */
  uint32_t n_tasks;
  uint32_t jit;   /* 1 = just-in-time launch, 0 = ahead-of-time        */
  uint32_t rows, cols; /* output tensor shape                          */
} mpk_export_op;

typedef struct mpk_export_task {
  uint32_t op;   /* index into ops, MPK_TASK_DUMMY_OP for a dummy task */
  uint32_t tile; /* tile index ib * tc + ic within the operator        */
  int32_t dep_event, trig_event; /* MPK_NO_EVENT if none               */
  int32_t worker; /* pre-assigned worker (AOT), -1 for JIT             */
  uint32_t jit;
} mpk_export_task;

typedef struct mpk_export_event {
  uint32_t required; /* notifications needed for activation                       */
  uint32_t first;    /* first launched task (index into the linearized task list) */
  uint32_t last;     /* one past the last launched task (empty range: == first)   */
  uint32_t flags;    /* bit 0: launches JIT tasks (handled by a scheduler)        */
} mpk_export_event;

enum {
  MPK_OP_EMBED = 0, MPK_OP_RMSNORM = 1, MPK_OP_LINEAR = 2, MPK_OP_ROPE = 3,
  MPK_OP_ATTN_PARTIAL = 4, MPK_OP_ATTN_MERGE = 5, MPK_OP_ADD = 6, MPK_OP_SWIGLU = 7,
  MPK_OP_GATEUP = 8, MPK_OP_ROUTER = 9, MPK_OP_EXPERT = 10, MPK_OP_COMBINE = 12, MPK_OP_ARGMAX = 13,
  MPK_OP_SERVE = 14
};

mpk_status mpk_graph_export(const mpk_graph *g, void *buf, size_t cap, size_t *need);

/* Per-task timeline of the LAST decode step of a graph compiled with MPK_DEBUG_TRACE (the
 * counterpart of the paper's run-time overhead accounting, Section 6.5 "kernel-launch
 * reduction").  buf: host u64 [n_tasks][12] in linearized task order, ticks of the 100 MHz device
 * wall clock unless noted: 0 task picked up, 1 dependent event seen, 2 input staged (linear and
 * attention tasks), 3 body finished (first wavefront), 4 triggering event notified, 5 worker
 * index (not a time), 6 first wavefront's stores completed, 7 all wavefronts' stores completed,
 * 8 multiply phase finished (matrix-core linear tasks), 10 attention: this task's partial result
 * combined over its wavefronts, 11 attention: partial result stored.  Slots a task kind does not
 * use stay 0.
 * Call after synchronising the stream.  buf == NULL returns the element count in *need. */
mpk_status mpk_graph_trace(mpk_graph *g, uint64_t *buf, size_t cap, size_t *need);

/* Mixture-of-experts graphs: the number of distinct experts the LAST decode step selected in each
 * layer (word 0 of each layer's meta-tensor, Section 6.4), i.e. how many experts' weights that
 * step streamed.  out: host u32 [n_layers].  Call after synchronising the stream; buf == NULL
 * returns the element count in *need.  INVALID_ARG for a dense or host_only graph. */
mpk_status mpk_graph_moe_active(mpk_graph *g, uint32_t *out, size_t cap, size_t *need);

/* Mixture-of-experts graphs, Section 6.4 (tasks re-balanced at run time from the meta-tensor):
 * which of the active experts' 16-row weight tiles -- laid end to end in ascending expert order,
 * n_active x tiles_per_expert of them -- expert task `task` of `n_tasks` works on in a step that
 * selected n_active distinct experts: tiles [*first, *last).  The shares are disjoint, in task
 * order, cover every tile, and are equal in cost rather than in tiles: an expert boundary inside
 * a share (a second job for the task) is charged like 8 tiles.  A pure function, the one the
 * kernels evaluate; no GPU is touched.  INVALID_ARG: a null pointer, n_tasks == 0, task >=
 * n_tasks or tiles_per_expert == 0. */
mpk_status mpk_moe_task_share(uint32_t n_active, uint32_t tiles_per_expert, uint32_t n_tasks,
                              uint32_t task, uint32_t *first, uint32_t *last);

/* Mixture-of-experts graphs: the routing decision of the LAST decode step (from each layer's
 * meta-tensor).  experts: host u32 [n_layers][batch][top_k], a token's experts in ascending index;
 * weights: host fp32, same shape, the renormalised combine weights; either may be NULL.  cap is in
 * elements; both NULL returns the element count in *need.  Call after synchronising the stream. */
mpk_status mpk_graph_moe_selection(mpk_graph *g, uint32_t *experts, float *weights, size_t cap,
                                   size_t *need);

/* One graph per representative batch size (Section 6.1, "Supporting runtime dynamism": task graphs
 * specialised for the powers of two up to the maximum batch size, the one that fits the current
 * batch is selected at run time).  mpk_compile_set compiles graphs for batch 1, 2, 4, ... below
 * cfg->batch and for cfg->batch itself; all of them share the weights and the ONE KV cache, which
 * is laid out for cfg->batch sequences (a smaller graph works on the first slots of it).
 * opts->kv_batch must be 0.  Errors as mpk_compile; on failure nothing is left allocated. */
typedef struct mpk_graph_set mpk_graph_set;
mpk_status mpk_compile_set(const mpk_model_config *cfg, const mpk_weight_ptrs *weights,
                           const mpk_kv_ptrs *kv, const mpk_compile_options *opts,
                           mpk_graph_set **out);
/* Number of graphs in the set; graph i (borrowed, ascending batch size, NULL if i is out of
 * range) for stats / status / export; the batch size of the graph that runs n_active sequences
 * (0 if n_active is 0 or above the maximum). */
uint32_t mpk_set_size(const mpk_graph_set *s);
mpk_graph *mpk_set_graph(mpk_graph_set *s, uint32_t i);
uint32_t mpk_set_batch_for(const mpk_graph_set *s, uint32_t n_active);
/* One decode step for the sequences in slots 0 .. n_active-1, on the smallest graph that holds
 * them (batch b = mpk_set_batch_for(s, n_active)).  Slots n_active .. b-1 are computed as padding:
 *   token_ids, positions : device int32, at least b entries, ALL valid (padding slots included:
 *                          their cache rows at positions[slot] are overwritten)
 *   logits_out           : device fp32 [b][vocab]; rows n_active .. b-1 belong to the padding
 * Otherwise as mpk_decode_step.  INVALID_ARG if n_active is 0 or above the maximum batch. */
mpk_status mpk_set_decode_step(mpk_graph_set *s, uint32_t n_active, const int32_t *token_ids,
                               const int32_t *positions, float *logits_out, void *stream);
void mpk_set_destroy(mpk_graph_set *s);

/* ----------------------------------------------------------------------------------------------
 * Paged KV cache and serving inside the task graph (Section 6.1, "supporting runtime dynamism").
 * -------------------------------------------------------------------------------------------- */

/* Give a graph compiled with kv_page_size (and without serving) the page table its attention
 * tasks read: device int32 [batch][max_seq / kv_page_size], entry [b][i] = page that holds rows
 * i * kv_page_size .. of sequence b.  Only entries for rows 0 .. positions[b] (+ the steps of a
 * multi-token launch) are read; an entry outside [0, kv_pages) is reported by mpk_graph_status
 * (MPK_ERR_DEVICE) and never dereferenced.  The pointer is kept, the contents may change between
 * launches.  Synchronous (a small copy); not while a launch of the graph is in flight. */
mpk_status mpk_graph_set_page_table(mpk_graph *g, const int32_t *page_table);

/* A server: the request queue, the slot table, the page tables and the free-page stack that the
 * graph's serving task (compile option serving = 1) works on, all in device memory.  Each decoding
 * iteration starts with that ONE task, which (1) removes completed requests, (2) admits arrivals,
 * (3) updates the KV-cache metadata the attention tasks then read (Section 6.1).  The paper fixes
 * no policy; this is the contract:
 *   - a request is a prompt and max_new_tokens; it ends with max_new_tokens produced tokens or with
 *     eos_token (kept as its last token).  Prompts go through the decode path, one token per
 *     iteration; the token sampled meanwhile is ignored.
 *   - retire: slots in ascending order; pages go back on the free stack in page-table order.
 *   - close ranks: the requests still running move, in order, to the lowest slots (a slot is
 *     metadata only; the rows stay in their pages), so running requests always fill slots 0..n-1.
 *   - admit: idle slots in ascending order take requests in arrival order; a request enters only
 *     when ceil((prompt_len + max_new_tokens - 1) / kv_page_size) pages are free and not promised
 *     to running requests; the first request that does not fit ends admission for the iteration.
 *   - a running slot pops a page when its position reaches a page boundary; an idle slot computes
 *     on token 0 at position 0 in a page of its own (pages 0 .. batch-1 are reserved for that).
 * Sampling is greedy (the graph's sampling operator). */
typedef struct mpk_serve_config {
  uint32_t struct_size;  /* = sizeof(mpk_serve_config)                                  */
  uint32_t max_requests; /* requests the server accepts over its lifetime (1 .. 2^20)   */
  uint32_t max_prompt;   /* longest prompt, in tokens (1 .. max_seq)                     */
  uint32_t max_new;      /* largest max_new_tokens of a request (1 .. max_seq)           */
  int32_t eos_token;     /* -1 = none                                                    */
} mpk_serve_config;
typedef struct mpk_server mpk_server;

/* Allocates and initialises the server's device state and attaches it to `g` (one server per
 * graph; destroy it before the graph).  Errors: INVALID_ARG, OOM, HIP. */
mpk_status mpk_serve_create(mpk_graph *g, const mpk_serve_config *cfg, mpk_server **out);
/* The same over a graph set compiled with serving = 1 (mpk_compile_set: a graph per power-of-two
 * batch size, Section 6.1): one server state shared by all graphs, sized for the largest batch.
 * Every mpk_serve_run then launches the graph of the smallest batch size that holds the requests
 * that can be in flight, min(largest batch, submitted - finished), where "finished" is what the
 * host has read back so far through mpk_serve_result or mpk_serve_state (a caller that never
 * reads back always runs the largest graph once enough requests were submitted). */
mpk_status mpk_serve_create_set(mpk_graph_set *set, const mpk_serve_config *cfg, mpk_server **out);
/* Batch size of the graph the last mpk_serve_run launched (0 before the first). */
uint32_t mpk_serve_last_batch(const mpk_server *s);
/* mpk_graph_status over every graph of the server (after the caller synchronised the stream). */
mpk_status mpk_serve_status(mpk_server *s);
/* Queue a request: prompt = HOST int32 [prompt_len] (copied before the call returns), tokens in
 * [0, vocab).  The request becomes visible to the serving task of launches issued on `stream`
 * after this call.  request_id (host, may be NULL) = arrival number, from 0.  INVALID_ARG when
 * the request could never be admitted (rows above max_seq, more pages than the pool can free). */
mpk_status mpk_serve_submit(mpk_server *s, const int32_t *prompt, uint32_t prompt_len,
                            uint32_t max_new_tokens, void *stream, uint32_t *request_id);
/* Run up to n_iterations decoding iterations (1 .. 65535) with no host round trip between them:
 * a launch of the single-step kernel per iteration, issued back to back (measured faster than the
 * alternative at every batch size: see greedy_loop) -- or ONE launch of the persistent kernel for
 * all of them when the graph was compiled with greedy_loop = 2 (and for graphs that fall back to
 * the generic kernels) -- or per-operator launches with MPK_LAUNCH_PER_OP.  Every iteration is the serving
 * task, one decode step of all slots, greedy sampling.  The kernel runs until its workload is done
 * (Section 5): the iteration whose serving task finds nothing running and nothing queued is the
 * call's last; launches queued behind it only settle the event counters and leave
 * (mpk_serve_state tells how many iterations have run; with MPK_LAUNCH_PER_OP all of them run).  Asynchronous on `stream`; launches of one server
 * must not overlap.  Errors as mpk_decode_steps; device errors through mpk_graph_status. */
mpk_status mpk_serve_run(mpk_server *s, uint32_t n_iterations, void *stream);
/* After the caller synchronised the stream: state (0 queued, 1 running, 2 done) and the tokens a
 * request has produced so far (tokens = HOST int32 [cap] or NULL; n_tokens = how many exist). */
mpk_status mpk_serve_result(mpk_server *s, uint32_t request_id, int32_t *tokens, size_t cap,
                            uint32_t *n_tokens, uint32_t *state);
/* After the caller synchronised the stream: the whole serving state as int32 words into buf
 * (HOST, cap words; *need = words required, nothing is written when cap is too small):
 *   [0] batch B  [1] blocks per sequence M  [2] free pages  [3] promised pages  [4] requests
 *   admitted  [5] requests submitted  [6] iterations run  [7] tokens produced, then
 *   slot_req[B] (-1 idle), slot_pos[B], slot_held[B], token[B] (what the last iteration
 *   sampled: the next iteration's serving task reads it there), position[B],
 *   page table [B][M] (-1 = none), free stack [kv_pages] (the first [2] entries, top last). */
mpk_status mpk_serve_state(mpk_server *s, int32_t *buf, size_t cap, size_t *need);
/* Device fp32 [batch][vocab]: the logits of the last iteration run (owned by the server). */
const float *mpk_serve_logits(const mpk_server *s);
void mpk_serve_destroy(mpk_server *s);

const char *mpk_last_error(void);
void mpk_graph_destroy(mpk_graph *g);

#ifdef __cplusplus
}
#endif
#endif /* MPK_H */
