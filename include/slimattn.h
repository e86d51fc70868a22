/*
 * libslimattn -- memory-efficient causal attention, forward and backward, over fine-grained
 * slices of variable-length packed samples, with separate forward and backward unit lists.
 * One MI355X (gfx950), hand-written HIP.  C ABI: plain pointers and sizes only.
 *
 * Problem statement (SlimPack, arxiv 2509.26246):
 *   - samples are cut into slices by exploiting causality (Balanced Packing & Asymmetric
 *     Partitioning Solver subsection); a slice is a run of consecutive query rows of one sample;
 *   - a scheduling unit (the paper's MicroPack) is a list of slices: consecutive slices of one
 *     long sample, whole short samples, or a mix (SlimPack System section);
 *   - the forward pass and the backward pass use different unit lists (Asymmetric Partition);
 *   - a slice's queries attend to the keys/values of every earlier slice of the same sample (the
 *     KV cache) and causally to the slice itself (PackFlow Pipeline Parallelism Scheduling);
 *   - the backward pass recomputes the scores from q, k and a saved row statistic (Asymmetric
 *     Cost Profile paragraph) and a slice's dK/dV collect contributions from every later slice
 *     (DAG simulator, inter-slice dependencies).
 *
 * Tensor layouts (token-major, packed): q, o, dO, dQ : [T, Hq, d];  k, v, dK, dV : [T, Hkv, d];
 * lse : [Hq, T] float.  Query head h uses KV head h / (Hq / Hkv).
 *
 * Pointer kinds are stated per argument: HOST = ordinary host memory, DEVICE = memory of the
 * current HIP device (allocated and owned by the caller; the library never frees it).
 *
 * Every function returns SLIMATTN_OK (0) or a negative SLIMATTN_E* code; nothing throws, aborts
 * or synchronises the device unless stated.  Compute calls are asynchronous on the given stream.
 */
#ifndef SLIMATTN_H
#define SLIMATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLIMATTN_OK       0
#define SLIMATTN_EINVAL  -1   /* null / misaligned pointer, unsupported head_dim, dtype, Hq % Hkv != 0, bad range */
#define SLIMATTN_ETABLE  -2   /* tables inconsistent (see slimattn_validate) */
#define SLIMATTN_ECAP    -3   /* an output array is too small */
#define SLIMATTN_EHIP    -4   /* a HIP call failed; code via slimattn_last_hip_error() */
#define SLIMATTN_ENOMEM  -5   /* host allocation failed */
#define SLIMATTN_EINFEASIBLE -7 /* slimattn_solve_partition: the token cap alone needs more units than allowed */
#define SLIMATTN_ESCRATCH -6  /* slimattn_bwd_static: the pack needs more scratch than the built-in array holds */

#define SLIMATTN_F32   0      /* q,k,v,o,dO,dQ,dK,dV are float; all arithmetic fp32 */
#define SLIMATTN_BF16  1      /* tensors are bf16; products on bf16 MFMA, fp32 accumulation and softmax */

/* One slice of one sample.  q_start is a global token index; kv_start is the first token of the
 * sample; kv_len = q_start + q_len - kv_start is the number of keys the slice can see. */
typedef struct slimattn_slice {
  int32_t sample, idx_in_sample, q_start, q_len, kv_start, kv_len, rsv0, rsv1;
} slimattn_slice;

/* Grouping policies of the host-side unit builder.  All are deterministic.  "Walk order": samples
 * by descending length (ties: lower index first; the paper sorts samples by descending forward
 * cost), each sample's slices ascending (forward) or descending (backward: first-in, last-out).
 * cost(slice) = w_quad * pairs + w_lin * q_len, pairs = visible (query, key) pairs. */
#define SLIMATTN_POLICY_ALL           0  /* one unit holding every slice in table order */
#define SLIMATTN_POLICY_PER_SAMPLE    1  /* one unit per sample; slices descend if backward != 0 */
#define SLIMATTN_POLICY_ROUND_ROBIN   2  /* slice t -> unit t mod m; units listed descending if descending != 0 */
#define SLIMATTN_POLICY_PREFIX_FILL   3  /* walk order; slice with cost interval [C, C+c) -> unit floor(m(2C+c)/(2W)),
                                            clamped to m-1: the paper's per-unit target W/m with a midpoint rule */
#define SLIMATTN_POLICY_TOKEN_CAP     4  /* walk order; next-fit, a unit is closed when the next slice would push it
                                            over `cap` query tokens */
#define SLIMATTN_POLICY_SEEDED_LPT    5  /* every slice of a multi-slice sample seeds its own unit; single-slice
                                            samples, in walk order, each join the currently cheapest unit */
#define SLIMATTN_POLICY_ISOLATE_FILL  6  /* slices with cost*m*theta_den >= theta_num*W become singleton units; the
                                            rest are PREFIX_FILLed into max(1, m - n_isolated) units; an isolated
                                            slice closes the unit that is open at its place in the walk */

typedef struct slimattn_policy {
  int32_t kind;
  int32_t m;            /* target number of units (ROUND_ROBIN, PREFIX_FILL, ISOLATE_FILL) */
  int64_t w_quad;       /* cost weights */
  int64_t w_lin;
  int32_t backward;     /* walk a sample's slices in descending order */
  int32_t descending;   /* ROUND_ROBIN: list each unit's slices in descending table order */
  int32_t cap;          /* TOKEN_CAP */
  int32_t m_min;        /* SEEDED_LPT: at least this many units before filling */
  int32_t theta_num, theta_den;   /* ISOLATE_FILL threshold as a fraction */
} slimattn_policy;

typedef struct slimattn_params {
  int32_t total_tokens;      /* T */
  int32_t n_q_heads;         /* Hq */
  int32_t n_kv_heads;        /* Hkv, divides Hq */
  int32_t head_dim;          /* d: 64 or 128 (bf16); 16, 32, 64 or 128 (f32); see slimattn_shape_supported */
  int32_t dtype;             /* SLIMATTN_F32 or SLIMATTN_BF16 */
  float   scale;             /* softmax scale applied to q.k */
  int32_t unit_lo, unit_hi;  /* run units [unit_lo, unit_hi) of the pass's list; unit_hi = -1 means all */
  int32_t flags;             /* SLIMATTN_FLAG_* */
} slimattn_params;

#define SLIMATTN_FLAG_PER_UNIT_LAUNCH 1  /* one launch per unit instead of one fused launch over the range */
#define SLIMATTN_FLAG_STATS_PREPASS   2  /* bf16 backward: row statistics (delta = dO . O) in a launch of their own instead of
                                          * inside the dQ kernel (what the library does by itself for very long samples) */

#define SLIMATTN_CHECK_FORWARD   0
#define SLIMATTN_CHECK_BACKWARD  1
#define SLIMATTN_CHECK_ORDER     2       /* also enforce the paper's pipeline order rules */

typedef struct slimattn_tables slimattn_tables;   /* opaque: host + device copies of all tables */

/* ---- host-side unit-descriptor builder (no GPU needed) ------------------------------------- */

/* Cut every sample into slices of `slice_size` rows from its start (last one may be short).
 * lengths HOST [n]; cu_out HOST [n+1] (cumulative starts); out HOST [cap]; n_slices HOST out.
 * ECAP if cap is too small (n_slices still receives the needed count); EINVAL on a length < 0
 * or slice_size < 1 or total tokens beyond int32. */
int slimattn_build_slices(const int32_t* lengths, int32_t n, int32_t slice_size, int32_t* cu_out,
                          slimattn_slice* out, int32_t cap, int32_t* n_slices);

/* Same, from explicit interior cut points: sample s is cut at bounds[bounds_ptr[s] .. bounds_ptr[s+1])
 * (strictly increasing, inside (0, L)).  All arrays HOST. */
int slimattn_build_slices_from_bounds(const int32_t* lengths, int32_t n, const int32_t* bounds_ptr,
                                      const int32_t* bounds, int32_t* cu_out, slimattn_slice* out,
                                      int32_t cap, int32_t* n_slices);

/* Group slices into units for one pass.  unit_ptr HOST [cap_units+1], unit_slices HOST [n_slices]
 * (CSR: unit u holds unit_slices[unit_ptr[u] .. unit_ptr[u+1])); empty units are dropped.
 * cu HOST [n+1].  ECAP if cap_units is too small; EINVAL on a bad policy. */
int slimattn_build_units(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                         const slimattn_policy* policy, int32_t* unit_ptr, int32_t* unit_slices,
                         int32_t cap_units, int32_t* n_units);

/* ---- partition solver (host only) ---------------------------------------------------------------- */

/* Parameters of slimattn_solve_partition.  A row that sees i + 1 keys costs w_quad * (i + 1) + w_lin in its
 * pass (the paper gives only the ratios: attention backward = 2.5 x forward, linear layers 2 x; e.g. forward
 * 2 / lambda, backward 5 / 2 lambda in units of 2*d*Hq flops). */
typedef struct slimattn_solver {
  int32_t m_fwd, m_bwd;                  /* at most this many forward / backward units */
  int64_t w_quad_fwd, w_lin_fwd;         /* forward cost weights  (0 .. 2^20, 0 .. 2^30) */
  int64_t w_quad_bwd, w_lin_bwd;         /* backward cost weights */
  int32_t granule;                       /* cuts fall on multiples of this many rows from a sample's start (>= 1) */
  int32_t token_cap_fwd, token_cap_bwd;  /* at most this many query rows per unit (0: no cap); a single granule may exceed it */
  int32_t max_slice;                     /* extra cuts every max_slice rows so that no slice is longer (0: none) */
} slimattn_solver;

/* Exact solution of the paper's Phase 2 problem in the form this library states it (Balanced Packing &
 * Asymmetric Partitioning Solver: per-unit target tau = W / m, long samples cut into slices over several units,
 * short ones packed, slice boundaries decided by the optimisation; Asymmetric Partition: a partition of its own
 * for the backward pass, same unit order).  Units are contiguous pieces of the walk (samples by descending
 * length, ties by index; rows upwards forward, downwards backward); the largest unit cost is minimised over all
 * cuts on granule boundaries, for each pass separately (bottlenecks[0] forward, [1] backward receive the optimum;
 * optional); the cuts returned close a unit only when the next granule would exceed that optimum or the token
 * cap.  The slice table (same record layout and order as slimattn_build_slices) is the union of both passes'
 * cuts; both unit lists are CSR over it and satisfy SLIMATTN_CHECK_ORDER.
 * All arrays HOST: lengths [n]; cu_out [n+1]; slices [cap_slices]; *_unit_ptr [cap_units+1]; *_unit_slices
 * [cap_slices].  ECAP if a capacity is too small (n_slices, n_fwd_units, n_bwd_units are still set);
 * EINFEASIBLE if the token cap needs more than m units; EINVAL on bad parameters. */
int slimattn_solve_partition(const int32_t* lengths, int32_t n, const slimattn_solver* sp, int32_t* cu_out,
                             slimattn_slice* slices, int32_t cap_slices, int32_t* n_slices, int32_t* fwd_unit_ptr,
                             int32_t* fwd_unit_slices, int32_t* n_fwd_units, int32_t* bwd_unit_ptr,
                             int32_t* bwd_unit_slices, int32_t* n_bwd_units, int32_t cap_units, int64_t* bottlenecks);

/* The optimum of the same problem for several candidate unit counts (the paper evaluates several MicroPack
 * counts m and keeps the best; Primitive Measurements and Search Space), computed by n_threads workers:
 * fwd_bottleneck[i], bwd_bottleneck[i] for m_list[i] (used for both passes; m_fwd / m_bwd of `sp` are
 * ignored); -1 where the token cap makes m_list[i] units infeasible.  All arrays HOST [n_m]. */
int slimattn_solve_bottlenecks(const int32_t* lengths, int32_t n, const slimattn_solver* sp, const int32_t* m_list,
                               int32_t n_m, int32_t n_threads, int64_t* fwd_bottleneck, int64_t* bwd_bottleneck);

/* ---- DAG-based pipeline simulator (host only) -------------------------------------------------------- */

#define SLIMATTN_ACTION_FWD     0
#define SLIMATTN_ACTION_BWD     1
#define SLIMATTN_EDGE_STAGE     0   /* inter-stage data dependency */
#define SLIMATTN_EDGE_SLICE     1   /* inter-slice data dependency (KV cache forward, KV gradients backward) */
#define SLIMATTN_EDGE_SCHEDULE  2   /* order of tasks on one stage */

/* Execution timeline on a task graph (paper: DAG resolution; Execution timeline calculation on the DAG):
 * Start(v) = max(0, Finish(u) over edges (u, v)), Finish(v) = Start(v) + weight[v], *total = max Finish, by
 * topological order and edge relaxation, O(V + E).  weight [n_vertices] >= 0 in any integer time unit; edges
 * as (edge_from[e], edge_to[e]) vertex indices; start, finish [n_vertices] out.  All arrays HOST.
 * ETABLE if the graph has a cycle (the schedule would deadlock); EINVAL on bad indices or negative weights. */
int slimattn_dag_timeline(int32_t n_vertices, const int64_t* weight, int32_t n_edges, const int32_t* edge_from,
                          const int32_t* edge_to, int64_t* start, int64_t* finish, int64_t* total);

/* Task graph of a 1F1B pipeline of n_stages stages over the given slice table and forward / backward unit lists
 * (paper: DAG-based pipeline representation -- vertices (stage, action, data unit), inter-stage, inter-slice and
 * schedule dependencies; PackFlow Pipeline Parallelism Scheduling -- units first-in first-out, a sample's
 * backward after all of its slices' forward, an extra forward unit while the next backward unit is not ready).
 * Vertex ids: forward task of unit u on stage s = s * n_fwd + u; backward task of unit v on stage s =
 * n_stages * n_fwd + s * n_bwd + v.  vertex [3 * cap_vertices] receives (stage, action, unit) per vertex, weight
 * [cap_vertices] the task times taken from fwd_cost [n_fwd] / bwd_cost [n_bwd] (the same on every stage);
 * edge_from, edge_to, edge_kind [cap_edges] the edges with their SLIMATTN_EDGE_* kind.  With asymmetric unit
 * lists a backward unit at the last stage depends on every forward unit it shares a slice with.  All arrays
 * HOST.  ECAP if a capacity is too small (n_vertices, n_edges are still set); ETABLE on inconsistent lists. */
int slimattn_dag_build_1f1b(const slimattn_slice* slices, int32_t n_slices, const int32_t* fwd_unit_ptr,
                            const int32_t* fwd_unit_slices, int32_t n_fwd, const int32_t* bwd_unit_ptr,
                            const int32_t* bwd_unit_slices, int32_t n_bwd, int32_t n_stages, const int64_t* fwd_cost,
                            const int64_t* bwd_cost, int32_t* vertex, int64_t* weight, int32_t cap_vertices,
                            int32_t* n_vertices, int32_t* edge_from, int32_t* edge_to, int32_t* edge_kind,
                            int32_t cap_edges, int32_t* n_edges);

/* Memory footprint over a timeline (paper: Memory footprint simulation -- allocation and release events are
 * simulated chronologically on the execution timeline).  Buffer b belongs to stage buf_stage[b], holds
 * buf_bytes[b] >= 0 bytes and is live from start[buf_alloc_vertex[b]] up to, not including,
 * finish[buf_free_vertex[b]] (at one instant releases come before allocations).  start, finish [n_vertices] as
 * slimattn_dag_timeline wrote them; stage_base [n_stages] the constant part of each stage (weights, optimizer
 * states), NULL for zero.  peak_bytes, peak_time [n_stages] out: the largest live size of the stage and the
 * earliest instant it is reached (0 if the stage has no live buffer).  All arrays HOST.
 * ETABLE if a buffer would be released before it is allocated; EINVAL on bad indices or negative sizes. */
int slimattn_dag_memory(int32_t n_vertices, const int64_t* start, const int64_t* finish, int32_t n_buffers,
                        const int32_t* buf_stage, const int64_t* buf_bytes, const int32_t* buf_alloc_vertex,
                        const int32_t* buf_free_vertex, int32_t n_stages, const int64_t* stage_base, int64_t* peak_bytes,
                        int64_t* peak_time);

/* The buffers of the graph slimattn_dag_build_1f1b makes of the same tables (same vertex ids), three per
 * (stage, slice) in this order (paper: Memory footprint simulation -- activations held from the forward task to
 * the corresponding backward task; KV cache and gradients managed per slice according to the schedule):
 *   activations   act_bytes_per_token x q_len, from the slice's forward task to its backward task;
 *   KV cache      kv_bytes_per_token x q_len, from the slice's forward task to the stage's last backward task
 *                 that reads it: the last unit holding a slice of the same sample at or after it;
 *   KV gradients  grad_bytes_per_token x q_len, from the first such backward task to the last (the rule of
 *                 slimattn_bwd_released_rows at slice granularity).
 * per_slice = 0 gives the sample-wise lifetimes to compare with: a sample's whole KV cache from its first
 * forward task to its last backward task, its gradients from its first backward task to its last.
 * buf_* [cap_buffers] out, *n_buffers = 3 * n_stages * n_slices.  All arrays HOST.  ECAP if cap_buffers is too
 * small (n_buffers is still set); ETABLE on inconsistent lists; EINVAL on bad arguments. */
int slimattn_dag_buffers_1f1b(const slimattn_slice* slices, int32_t n_slices, const int32_t* fwd_unit_ptr,
                              const int32_t* fwd_unit_slices, int32_t n_fwd, const int32_t* bwd_unit_ptr,
                              const int32_t* bwd_unit_slices, int32_t n_bwd, int32_t n_stages, int64_t act_bytes_per_token,
                              int64_t kv_bytes_per_token, int64_t grad_bytes_per_token, int32_t per_slice, int32_t* buf_stage,
                              int64_t* buf_bytes, int32_t* buf_alloc_vertex, int32_t* buf_free_vertex, int32_t cap_buffers,
                              int32_t* n_buffers);

/* ---- search over the number of units (host only) ----------------------------------------------------- */

/* How a candidate is priced (paper: Primitive Measurements and Search Space -- runtimes estimated from the
 * theoretical cost with utilisations calibrated by preliminary benchmarks; DAG-based Pipeline Simulator).
 * Task time of a unit = fixed + cost * num / den (integer division), cost = w_quad * pairs + w_lin * rows of
 * its slices with the pass's weights of slimattn_solver; any time unit.  Bytes per token as in
 * slimattn_dag_buffers_1f1b (per-slice lifetimes).  stage_bytes_cap > 0: a candidate whose worst stage's peak
 * exceeds it is not chosen. */
typedef struct slimattn_search {
  int32_t n_stages;
  int32_t pad0;
  int64_t fwd_fixed, fwd_num, fwd_den;
  int64_t bwd_fixed, bwd_num, bwd_den;
  int64_t act_bytes_per_token, kv_bytes_per_token, grad_bytes_per_token;
  int64_t stage_bytes_cap;
} slimattn_search;

/* Candidate unit counts m = i * n_stages <= m_max for i = 1, 2, 3, 4, 6, 8, 12, 16, 24, ... (paper: Primitive
 * Measurements and Search Space -- m quantised to multiples of the pipeline width, i sampled on a roughly
 * logarithmic grid; the grid itself is this build's: the powers of two and the values halfway between).
 * out [cap] ascending, *n_out the count (ECAP if cap is too small; the count is still set).  HOST. */
int slimattn_candidate_unit_counts(int32_t n_stages, int32_t m_max, int32_t* out, int32_t cap, int32_t* n_out);

/* For each candidate m_list[i] (used as the unit count of both passes; m_fwd / m_bwd of `sp` are ignored):
 * the exact partition (slimattn_solve_partition), its units priced by `ss`, through the 1F1B graph of
 * ss->n_stages stages (slimattn_dag_build_1f1b, slimattn_dag_timeline) and the memory footprint
 * (slimattn_dag_buffers_1f1b, slimattn_dag_memory): t_total[i] the simulated iteration time, peak_bytes[i]
 * the worst stage's peak; both -1 where the token cap makes m_list[i] units infeasible.  *best = index of the
 * candidate with the smallest t_total among those within stage_bytes_cap (ties: the earlier entry), -1 if
 * none (paper: Balanced Packing & Asymmetric Partitioning Solver -- several MicroPack counts are evaluated
 * and the best kept).  Candidates are evaluated by n_threads workers.  All arrays HOST [n_m]. */
int slimattn_search_unit_count(const int32_t* lengths, int32_t n, const slimattn_solver* sp, const slimattn_search* ss,
                               const int32_t* m_list, int32_t n_m, int32_t n_threads, int64_t* t_total, int64_t* peak_bytes,
                               int32_t* best);

/* Checks tables against the rules of the paper's PackFlow Pipeline Parallelism Scheduling section (slice order
 * within a sample preserved in the forward pass, backward first-in last-out) and of the MicroPack definition
 * (SlimPack System).  Structural rules (always): cu starts at 0 and is non-decreasing; the slices of a sample appear
 * in ascending order in the table, are non-empty and tile [0, L) exactly; kv_start/kv_len agree
 * with cu; unit_ptr is a valid CSR over unit_slices; every slice is in exactly one unit.
 * With SLIMATTN_CHECK_ORDER in `mode`: along a sample the unit index never decreases with the
 * slice index (forward) / never increases (SLIMATTN_CHECK_BACKWARD), and inside a unit a sample's
 * slices are adjacent in that order.  Returns OK or ETABLE; *rule (optional, HOST) receives a
 * static string naming the first violated rule.  All arrays HOST. */
int slimattn_validate(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                      const int32_t* unit_ptr, const int32_t* unit_slices, int32_t n_units, int mode,
                      const char** rule);

/* Visible (query, key) pairs of a slice, and the forward/backward flop counts the paper's
 * 1 : 2.5 ratio rests on: 2 resp. 5 tile products of 2*d*Hq flops per pair. */
int64_t slimattn_slice_pairs(const slimattn_slice* s);
int64_t slimattn_flops_fwd(int64_t pairs, int32_t head_dim, int32_t n_q_heads);
int64_t slimattn_flops_bwd(int64_t pairs, int32_t head_dim, int32_t n_q_heads);

/* ---- tables on the device -------------------------------------------------------------------- */

/* The device-side form of the paper's scheduling input (SlimPack System: MicroPacks as lists of slices;
 * Asymmetric Partition: one list per pass).  Validates (structural rules, both lists), derives the private tile work-lists and copies
 * everything to the current device with one synchronous upload.  All inputs HOST; they are copied.
 * *out receives a handle to free with slimattn_tables_destroy.  ETABLE / EHIP / ENOMEM. */
int slimattn_tables_create(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                           const int32_t* fwd_unit_ptr, const int32_t* fwd_unit_slices, int32_t n_fwd_units,
                           const int32_t* bwd_unit_ptr, const int32_t* bwd_unit_slices, int32_t n_bwd_units,
                           slimattn_tables** out);
/* The same with the upload queued on `stream` (use_stream != 0; NULL = the default stream) instead of a
 * synchronous copy: the host returns without waiting (the paper overlaps the solver with data loading so that
 * the compute stream never waits for a packing plan; Zero-Overhead Runtime Integration), and compute calls
 * queued on the same stream afterwards see the tables.  A compute call on another stream must be ordered after
 * the upload by the caller.  The handle keeps a pinned staging copy until it is destroyed. */
int slimattn_tables_create_async(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                                 const int32_t* fwd_unit_ptr, const int32_t* fwd_unit_slices, int32_t n_fwd_units,
                                 const int32_t* bwd_unit_ptr, const int32_t* bwd_unit_slices, int32_t n_bwd_units,
                                 void* stream, int use_stream, slimattn_tables** out);
void slimattn_tables_destroy(slimattn_tables* t);

/* Counts held by a handle: what = 0 tokens, 1 samples, 2 slices, 3 forward units, 4 backward units,
 * 5..8: 256-row key tiles of the whole-list scope whose dK/dV work is divided among several blocks
 * when the launch has 1, 2, 4, >= 8 KV heads (heavy-tile balancing; informational). */
int64_t slimattn_tables_count(const slimattn_tables* t, int what);

/* Bytes of DEVICE scratch slimattn_bwd needs (fp32 dK/dV accumulators, the per-row statistics in
 * fp32 and as bf16 triples, partial tiles of divided key tiles).  Its contents need no initialisation. */
size_t slimattn_bwd_workspace_bytes(const slimattn_tables* t, int32_t n_q_heads, int32_t n_kv_heads,
                                    int32_t head_dim);

/* ---- compute ------------------------------------------------------------------------------- */

/* Whether slimattn_fwd / slimattn_bwd accept a pack of this shape (host only; what they check themselves).
 * bf16: one sample's rows must stay below 2 GiB (max_sample_len * Hq * d * 2 < 2^31: tiles are addressed by
 * 32-bit offsets from the sample's or the key tile's first row), and total_tokens * Hq * 16 < 2^31 (row
 * statistics); the pack as a whole may exceed 2 GiB per tensor.  OK or EINVAL. */
int slimattn_shape_supported(int64_t total_tokens, int32_t max_sample_len, int32_t n_q_heads, int32_t n_kv_heads,
                             int32_t head_dim, int32_t dtype);

/* Forward over units [unit_lo, unit_hi) of the forward list (paper: PackFlow Pipeline Parallelism
 * Scheduling, slice-level causal attention with a KV cache): for every query row i of every slice in
 * those units and every head, S_ij = scale * q_i . k_j over the sample's keys j <= i,
 * lse_i = log sum_j exp S_ij, o_i = sum_j exp(S_ij - lse_i) v_j.
 * Incremental use: the call reads the q rows of the range's slices and, per sample, the k/v rows from the
 * sample's start to the last of those rows -- nothing else; rows of other units may hold anything (their
 * K/V need not exist yet), and o/lse rows of slices outside the range are not written.  A runtime can
 * therefore call it one unit at a time as K/V arrive slice by slice.
 * q, k, v DEVICE (read), o, lse DEVICE (written), 16-byte aligned.
 * stream: a hipStream_t (NULL = default stream).  Allocates nothing, does not synchronise, issues kernel
 * launches only (no memset, no copy): the call -- and slimattn_bwd likewise -- may be recorded by a stream
 * capture into a HIP graph, with slimattn_profile_enable off (its events do not belong in a capture). */
int slimattn_fwd(const slimattn_params* p, const void* q, const void* k, const void* v,
                 const slimattn_tables* t, void* o, float* lse, void* stream);

/* Backward over units [unit_lo, unit_hi) of the backward list, with the scores recomputed from q, k
 * and lse (paper: Asymmetric Cost Profile -- the recomputation is why backward costs 2.5 x forward;
 * Asymmetric Partition -- hence a unit list of its own): P_ij = exp(S_ij - lse_i), dP_ij = dO_i . v_j,
 * delta_i = dO_i . o_i, dS_ij = P_ij (dP_ij - delta_i); dQ_i = scale sum_j dS_ij k_j for the rows of the
 * range's slices; dK_j += scale sum_i dS_ij q_i and dV_j += sum_i P_ij dO_i over those rows i >= j and
 * over the query heads of j's group, in a fixed order (no float atomics; bitwise repeatable).
 * A key row collects from every later slice of its sample (paper: DAG-based pipeline representation,
 * inter-slice dependencies), i.e. possibly from several units.  Units must be run in list order, each
 * exactly once, over one or several calls that share `workspace`: the first unit that reaches a key row
 * starts its sum (nothing has to be cleared beforehand), later ones continue it in fp32 in the workspace, and
 * the last one writes dK/dV in the output type -- so a row's gradient is final as soon as its last
 * contributor has run (slimattn_bwd_released_rows), not only at the end of the list.
 * Incremental use: the call reads q, dO, o, lse rows of the range's slices and the k/v rows of their
 * samples up to those rows -- nothing else; dO, o, lse of other units may hold anything.
 * q, k, v, o, lse, dO DEVICE (read); dQ, dK, dV DEVICE (written); workspace DEVICE of at least
 * slimattn_bwd_workspace_bytes().  Allocates nothing, does not synchronise. */
int slimattn_bwd(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o,
                 const float* lse, const void* dO, const slimattn_tables* t, void* dQ, void* dK,
                 void* dV, void* workspace, void* stream);

/* Key rows whose dK/dV become final with backward unit `unit` (when the units before it have run): ranges
 * [ranges[2i], ranges[2i+1]) of global token indices, ascending, n_ranges of them -- per sample, the rows
 * between the last query row any later unit holds and the last query row this unit holds (paper: Memory
 * footprint simulation -- KV gradients are managed per slice).  Over all units the ranges partition
 * [0, T).  HOST arrays; ECAP if cap < n_ranges (n_ranges is still set). */
int slimattn_bwd_released_rows(const slimattn_tables* t, int32_t unit, int32_t* ranges, int32_t cap, int32_t* n_ranges);

/* For callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same computation, arguments,
 * unit ranges and flags as slimattn_bwd, with the workspace taken from an array built into the library
 * (SLIMATTN_STATIC_SCRATCH_BYTES of device memory per GPU the library runs on, held until the process
 * ends; its address is looked up once per device, by slimattn_tables_create or by the first call).  The call
 * allocates nothing and frees nothing.  SLIMATTN_ESCRATCH when slimattn_bwd_workspace_bytes() for this
 * pack exceeds the array (nothing is launched).  Every call on a GPU uses that GPU's one array, which keeps
 * what the last call left: a call with unit_lo == 0 clears what must start at zero, as slimattn_bwd does,
 * and calls that overlap in time on one GPU (two streams, two threads) race on it -- serialise them.  A
 * unit list split over several calls must not be interleaved with calls for another pack. */
#define SLIMATTN_STATIC_SCRATCH_BYTES (64u << 20)
int slimattn_bwd_static(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o,
                        const float* lse, const void* dO, const slimattn_tables* t, void* dQ, void* dK,
                        void* dV, void* stream);

/* ---- measurement aid --------------------------------------------------------------------------- */

/* Kernel classes reported by slimattn_profile_read. */
#define SLIMATTN_K_FWD       0
#define SLIMATTN_K_DELTA     1
#define SLIMATTN_K_DQ        2
#define SLIMATTN_K_DKDV      3
#define SLIMATTN_K_REDUCE    4          /* the reduction of divided key tiles */
#define SLIMATTN_K_UNUSED    5          /* (no kernel; kept so that class numbers stay put) */
#define SLIMATTN_K_FWD_CALL  6          /* a whole slimattn_fwd call, first launch to last, on the caller's stream */
#define SLIMATTN_K_BWD_CALL  7          /* a whole slimattn_bwd call, likewise (includes the gaps between its launches) */
#define SLIMATTN_K_COUNT     8

/* Per-kernel timing for benchmarks (the paper calibrates its simulator from such primitive
 * measurements, Primitive Measurements and Search Space; its Workload Balance Studies compare the
 * forward and backward time of each scheduling unit).  max_launches > 0: create that many
 * HIP event pairs on the current device; from then on every kernel launch made by slimattn_fwd /
 * slimattn_bwd is bracketed by two events recorded on the launch's own stream.  A launch that finds
 * the pool used up runs untimed and is counted as dropped.  max_launches == 0: stop and destroy the
 * events.  Not thread-safe; one device. */
int slimattn_profile_enable(int32_t max_launches);

/* Waits for the recorded events, adds up elapsed milliseconds and launch counts per kernel class
 * into ms[SLIMATTN_K_COUNT] and launches[SLIMATTN_K_COUNT] (HOST), and rewinds the pool.  Returns
 * SLIMATTN_ECAP (the sums are still written) when launches were dropped since the last read. */
int slimattn_profile_read(double* ms, int64_t* launches);

/* The same per launch, in launch order: kernel class, pass (0 forward, 1 backward), unit index in that
 * pass's list (-1: the launch covered a whole range or is not tied to a unit) and milliseconds.  All
 * arrays HOST [cap]; *n_launches receives the number recorded, *dropped (optional) the number that found
 * the pool used up.  ECAP when cap is too small (nothing is consumed); rewinds the pool on success. */
int slimattn_profile_read_launches(int32_t cap, int32_t* cls, int32_t* pass, int32_t* unit, float* ms,
                                   int32_t* n_launches, int64_t* dropped);

const char* slimattn_strerror(int code);
int slimattn_last_hip_error(void);       /* hipError_t of the last EHIP on this thread */
int slimattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SLIMATTN_H */
