// DAG-based pipeline simulator: execution timeline on a task graph, and the generator of that graph for a
// 1F1B pipeline over scheduling units whose forward and backward lists differ.  Pure host C++, integers only.
//
// Paper (DAG-based Pipeline Simulator): a vertex is a task (model_id = pipeline stage, action F or B, data_id =
// unit); its weight is the task's time; edges are data dependencies -- inter-stage (a unit flows down the stages
// in the forward pass and back up in the backward pass) and inter-slice (the forward of a slice needs the KV
// cache of the earlier slices of its sample, its backward the KV gradients of the later ones) -- and schedule
// dependencies (the order in which a stage executes its tasks: 1F1B fills the pipeline with forwards,
// alternates one forward and one backward, then drains).  DAG resolution: Start(v) = max(0, Finish(u) over
// edges (u, v)), Finish(v) = Start(v) + w(v), total = max Finish, by topological order and edge relaxation
// in O(V + E) (Execution timeline calculation on the DAG).
//
// With asymmetric partitioning the forward and backward unit lists group the slices differently, so "the same
// data unit" of the paper's chain at the last stage becomes: backward unit v waits for every forward unit that
// shares a slice with it.  A stage runs backward unit v only once all forward units holding slices of v's
// samples have been issued on that stage (the paper's rule that a sample's backward starts after all of its
// slices' forward passes); while the next backward unit is not ready the stage issues another forward unit
// (PackFlow section: an extra forward MicroPack is injected).
//
// The same timeline carries the memory footprint (Memory footprint simulation): allocation and release events at
// task starts and finishes, walked chronologically per stage; the 1F1B generator's buffers are each slice's
// activations, KV cache and KV gradients.
#include "internal.h"

#include <algorithm>
#include <climits>
#include <vector>

extern "C" {

int slimattn_dag_timeline(int32_t n_vertices, const int64_t* weight, int32_t n_edges, const int32_t* edge_from,
                          const int32_t* edge_to, int64_t* start, int64_t* finish, int64_t* total) {
  if (n_vertices < 0 || n_edges < 0 || (n_vertices > 0 && (!weight || !start || !finish)) || (n_edges > 0 && (!edge_from || !edge_to)) || !total)
    return SLIMATTN_EINVAL;
  for (int32_t e = 0; e < n_edges; ++e)
    if (edge_from[e] < 0 || edge_from[e] >= n_vertices || edge_to[e] < 0 || edge_to[e] >= n_vertices) return SLIMATTN_EINVAL;
  for (int32_t v = 0; v < n_vertices; ++v)
    if (weight[v] < 0) return SLIMATTN_EINVAL;
  // adjacency in CSR form, in-degrees
  std::vector<int32_t> first(n_vertices + 1, 0), indeg(n_vertices, 0), adj(n_edges);
  for (int32_t e = 0; e < n_edges; ++e) { first[edge_from[e] + 1]++; indeg[edge_to[e]]++; }
  for (int32_t v = 0; v < n_vertices; ++v) first[v + 1] += first[v];
  {
    std::vector<int32_t> fill(first.begin(), first.end() - 1);
    for (int32_t e = 0; e < n_edges; ++e) adj[fill[edge_from[e]]++] = edge_to[e];
  }
  for (int32_t v = 0; v < n_vertices; ++v) start[v] = 0;
  // topological order by repeatedly taking vertices without unprocessed predecessors; each vertex is
  // finished when taken and relaxes its successors' start times
  std::vector<int32_t> ready;
  ready.reserve(n_vertices);
  for (int32_t v = 0; v < n_vertices; ++v)
    if (indeg[v] == 0) ready.push_back(v);
  int64_t t_total = 0;
  size_t done = 0;
  while (done < ready.size()) {
    const int32_t u = ready[done++];
    finish[u] = start[u] + weight[u];
    t_total = std::max(t_total, finish[u]);
    for (int32_t i = first[u]; i < first[u + 1]; ++i) {
      const int32_t v = adj[i];
      start[v] = std::max(start[v], finish[u]);
      if (--indeg[v] == 0) ready.push_back(v);
    }
  }
  if ((int32_t)done != n_vertices) return SLIMATTN_ETABLE;      // a cycle: the schedule would deadlock
  *total = t_total;
  return SLIMATTN_OK;
}

int slimattn_dag_build_1f1b(const slimattn_slice* slices, int32_t n_slices, const int32_t* fwd_unit_ptr,
                            const int32_t* fwd_unit_slices, int32_t n_fwd, const int32_t* bwd_unit_ptr,
                            const int32_t* bwd_unit_slices, int32_t n_bwd, int32_t n_stages, const int64_t* fwd_cost,
                            const int64_t* bwd_cost, int32_t* vertex, int64_t* weight, int32_t cap_vertices, int32_t* n_vertices,
                            int32_t* edge_from, int32_t* edge_to, int32_t* edge_kind, int32_t cap_edges, int32_t* n_edges) {
  if (n_slices < 0 || n_fwd < 0 || n_bwd < 0 || n_stages < 1 || !fwd_unit_ptr || !bwd_unit_ptr || !n_vertices || !n_edges ||
      (n_slices > 0 && (!slices || !fwd_unit_slices || !bwd_unit_slices)) || (n_fwd > 0 && !fwd_cost) || (n_bwd > 0 && !bwd_cost))
    return SLIMATTN_EINVAL;
  if (fwd_unit_ptr[n_fwd] != n_slices || bwd_unit_ptr[n_bwd] != n_slices) return SLIMATTN_ETABLE;
  int32_t n_samples = 0;
  for (int32_t t = 0; t < n_slices; ++t) {
    if (slices[t].sample < 0) return SLIMATTN_ETABLE;
    n_samples = std::max(n_samples, slices[t].sample + 1);
  }
  std::vector<int32_t> fwd_of(n_slices, -1), bwd_of(n_slices, -1);
  for (int32_t u = 0; u < n_fwd; ++u)
    for (int32_t i = fwd_unit_ptr[u]; i < fwd_unit_ptr[u + 1]; ++i) {
      if (fwd_unit_slices[i] < 0 || fwd_unit_slices[i] >= n_slices || fwd_of[fwd_unit_slices[i]] != -1) return SLIMATTN_ETABLE;
      fwd_of[fwd_unit_slices[i]] = u;
    }
  for (int32_t v = 0; v < n_bwd; ++v)
    for (int32_t i = bwd_unit_ptr[v]; i < bwd_unit_ptr[v + 1]; ++i) {
      if (bwd_unit_slices[i] < 0 || bwd_unit_slices[i] >= n_slices || bwd_of[bwd_unit_slices[i]] != -1) return SLIMATTN_ETABLE;
      bwd_of[bwd_unit_slices[i]] = v;
    }
  // slices of each sample by index in the sample
  std::vector<std::vector<int32_t>> of_sample(n_samples);
  for (int32_t t = 0; t < n_slices; ++t) of_sample[slices[t].sample].push_back(t);
  for (auto& ts : of_sample) std::sort(ts.begin(), ts.end(), [&](int32_t a, int32_t b) { return slices[a].idx_in_sample < slices[b].idx_in_sample; });

  const int64_t nv = (int64_t)n_stages * (n_fwd + n_bwd);
  *n_vertices = (int32_t)nv;
  auto F = [&](int32_t s, int32_t u) { return s * n_fwd + u; };
  auto B = [&](int32_t s, int32_t v) { return n_stages * n_fwd + s * n_bwd + v; };

  std::vector<int32_t> ef, et, ek;
  auto edge = [&](int32_t a, int32_t b, int32_t kind) { ef.push_back(a); et.push_back(b); ek.push_back(kind); };
  auto unique_pairs = [](std::vector<std::pair<int32_t, int32_t>>& v) {
    std::sort(v.begin(), v.end());
    v.erase(std::unique(v.begin(), v.end()), v.end());
  };
  // inter-stage: forward units down the stages, backward units up, and at the last stage every backward unit
  // after the forward units that share a slice with it
  for (int32_t s = 0; s + 1 < n_stages; ++s)
    for (int32_t u = 0; u < n_fwd; ++u) edge(F(s, u), F(s + 1, u), SLIMATTN_EDGE_STAGE);
  {
    std::vector<std::pair<int32_t, int32_t>> fb;
    for (int32_t t = 0; t < n_slices; ++t) fb.emplace_back(fwd_of[t], bwd_of[t]);
    unique_pairs(fb);
    for (const auto& p : fb) edge(F(n_stages - 1, p.first), B(n_stages - 1, p.second), SLIMATTN_EDGE_STAGE);
  }
  for (int32_t s = n_stages - 1; s > 0; --s)
    for (int32_t v = 0; v < n_bwd; ++v) edge(B(s, v), B(s - 1, v), SLIMATTN_EDGE_STAGE);
  // inter-slice, on every stage: consecutive slices of a sample in different units
  {
    std::vector<std::pair<int32_t, int32_t>> ff, bb;
    for (const auto& ts : of_sample)
      for (size_t i = 0; i + 1 < ts.size(); ++i) {
        if (fwd_of[ts[i]] != fwd_of[ts[i + 1]]) ff.emplace_back(fwd_of[ts[i]], fwd_of[ts[i + 1]]);     // KV cache of the earlier slice
        if (bwd_of[ts[i]] != bwd_of[ts[i + 1]]) bb.emplace_back(bwd_of[ts[i + 1]], bwd_of[ts[i]]);     // KV gradients of the later slice
      }
    unique_pairs(ff);
    unique_pairs(bb);
    for (int32_t s = 0; s < n_stages; ++s) {
      for (const auto& p : ff) edge(F(s, p.first), F(s, p.second), SLIMATTN_EDGE_SLICE);
      for (const auto& p : bb) edge(B(s, p.first), B(s, p.second), SLIMATTN_EDGE_SLICE);
    }
  }
  // schedule: each stage's order of tasks.  need[v] = number of forward units that must have been issued before
  // backward unit v: all units holding a slice of one of v's samples.
  std::vector<int32_t> last_fwd_of_sample(n_samples, -1), need(n_bwd, 0);
  for (int32_t t = 0; t < n_slices; ++t) last_fwd_of_sample[slices[t].sample] = std::max(last_fwd_of_sample[slices[t].sample], fwd_of[t]);
  for (int32_t t = 0; t < n_slices; ++t) need[bwd_of[t]] = std::max(need[bwd_of[t]], last_fwd_of_sample[slices[t].sample] + 1);
  for (int32_t s = 0; s < n_stages; ++s) {
    std::vector<int32_t> order;
    int32_t i = 0, j = 0;
    const int32_t warm = std::min(n_stages - 1 - s, n_fwd);
    for (; i < warm; ++i) order.push_back(F(s, i));
    while (i < n_fwd) {                               // steady state: one forward, then one backward if it is ready
      order.push_back(F(s, i++));
      if (j < n_bwd && need[j] <= i) order.push_back(B(s, j++));
    }
    for (; j < n_bwd; ++j) order.push_back(B(s, j));   // cool-down
    for (size_t x = 0; x + 1 < order.size(); ++x) edge(order[x], order[x + 1], SLIMATTN_EDGE_SCHEDULE);
  }
  *n_edges = (int32_t)ef.size();
  if (nv > cap_vertices || (int64_t)ef.size() > cap_edges) return SLIMATTN_ECAP;
  if (nv > 0 && (!vertex || !weight)) return SLIMATTN_EINVAL;
  if (!ef.empty() && (!edge_from || !edge_to || !edge_kind)) return SLIMATTN_EINVAL;
  for (int32_t s = 0; s < n_stages; ++s) {
    for (int32_t u = 0; u < n_fwd; ++u) {
      const int32_t id = F(s, u);
      vertex[3 * id] = s; vertex[3 * id + 1] = SLIMATTN_ACTION_FWD; vertex[3 * id + 2] = u;
      weight[id] = fwd_cost[u];
    }
    for (int32_t v = 0; v < n_bwd; ++v) {
      const int32_t id = B(s, v);
      vertex[3 * id] = s; vertex[3 * id + 1] = SLIMATTN_ACTION_BWD; vertex[3 * id + 2] = v;
      weight[id] = bwd_cost[v];
    }
  }
  for (size_t e = 0; e < ef.size(); ++e) { edge_from[e] = ef[e]; edge_to[e] = et[e]; edge_kind[e] = ek[e]; }
  return SLIMATTN_OK;
}

// Memory footprint over a timeline (paper: Memory footprint simulation).  Every buffer is an allocation event at
// the start of one task and a release event at the finish of another; the events of a stage are walked in time
// order, releases before allocations at equal instants, and the largest running sum is the stage's peak.
int slimattn_dag_memory(int32_t n_vertices, const int64_t* start, const int64_t* finish, int32_t n_buffers,
                        const int32_t* buf_stage, const int64_t* buf_bytes, const int32_t* buf_alloc_vertex,
                        const int32_t* buf_free_vertex, int32_t n_stages, const int64_t* stage_base, int64_t* peak_bytes,
                        int64_t* peak_time) {
  if (n_vertices < 0 || n_buffers < 0 || n_stages < 0 || (n_vertices > 0 && (!start || !finish)) ||
      (n_buffers > 0 && (!buf_stage || !buf_bytes || !buf_alloc_vertex || !buf_free_vertex)) || (n_stages > 0 && (!peak_bytes || !peak_time)))
    return SLIMATTN_EINVAL;
  struct Event { int64_t time; int32_t kind; int64_t bytes; };     // kind 0 = release, 1 = allocation
  std::vector<std::vector<Event>> events(n_stages);
  for (int32_t b = 0; b < n_buffers; ++b) {
    const int32_t a = buf_alloc_vertex[b], f = buf_free_vertex[b];
    if (buf_stage[b] < 0 || buf_stage[b] >= n_stages || a < 0 || a >= n_vertices || f < 0 || f >= n_vertices || buf_bytes[b] < 0) return SLIMATTN_EINVAL;
    if (finish[f] < start[a]) return SLIMATTN_ETABLE;               // released before it exists
    if (finish[f] == start[a]) continue;                            // never live
    events[buf_stage[b]].push_back({start[a], 1, buf_bytes[b]});
    events[buf_stage[b]].push_back({finish[f], 0, buf_bytes[b]});
  }
  for (int32_t s = 0; s < n_stages; ++s) {
    auto& ev = events[s];
    std::sort(ev.begin(), ev.end(), [](const Event& x, const Event& y) { return x.time != y.time ? x.time < y.time : x.kind < y.kind; });
    int64_t live = 0, best = 0, at = 0;
    for (size_t i = 0; i < ev.size(); ++i) {
      live += ev[i].kind ? ev[i].bytes : -ev[i].bytes;
      // the sum counts once all events of an instant are in
      if ((i + 1 == ev.size() || ev[i + 1].time != ev[i].time) && live > best) { best = live; at = ev[i].time; }
    }
    peak_bytes[s] = (stage_base ? stage_base[s] : 0) + best;
    peak_time[s] = at;
  }
  return SLIMATTN_OK;
}

int slimattn_dag_buffers_1f1b(const slimattn_slice* slices, int32_t n_slices, const int32_t* fwd_unit_ptr,
                              const int32_t* fwd_unit_slices, int32_t n_fwd, const int32_t* bwd_unit_ptr,
                              const int32_t* bwd_unit_slices, int32_t n_bwd, int32_t n_stages, int64_t act_bytes_per_token,
                              int64_t kv_bytes_per_token, int64_t grad_bytes_per_token, int32_t per_slice, int32_t* buf_stage,
                              int64_t* buf_bytes, int32_t* buf_alloc_vertex, int32_t* buf_free_vertex, int32_t cap_buffers,
                              int32_t* n_buffers) {
  if (n_slices < 0 || n_fwd < 0 || n_bwd < 0 || n_stages < 1 || !fwd_unit_ptr || !bwd_unit_ptr || !n_buffers ||
      (n_slices > 0 && (!slices || !fwd_unit_slices || !bwd_unit_slices)) || act_bytes_per_token < 0 || kv_bytes_per_token < 0 ||
      grad_bytes_per_token < 0)
    return SLIMATTN_EINVAL;
  if (fwd_unit_ptr[n_fwd] != n_slices || bwd_unit_ptr[n_bwd] != n_slices) return SLIMATTN_ETABLE;
  std::vector<int32_t> fwd_of(n_slices, -1), bwd_of(n_slices, -1);
  for (int32_t u = 0; u < n_fwd; ++u)
    for (int32_t i = fwd_unit_ptr[u]; i < fwd_unit_ptr[u + 1]; ++i) {
      if (fwd_unit_slices[i] < 0 || fwd_unit_slices[i] >= n_slices || fwd_of[fwd_unit_slices[i]] != -1) return SLIMATTN_ETABLE;
      fwd_of[fwd_unit_slices[i]] = u;
    }
  for (int32_t v = 0; v < n_bwd; ++v)
    for (int32_t i = bwd_unit_ptr[v]; i < bwd_unit_ptr[v + 1]; ++i) {
      if (bwd_unit_slices[i] < 0 || bwd_unit_slices[i] >= n_slices || bwd_of[bwd_unit_slices[i]] != -1) return SLIMATTN_ETABLE;
      bwd_of[bwd_unit_slices[i]] = v;
    }
  int32_t n_samples = 0;
  for (int32_t t = 0; t < n_slices; ++t) {
    if (slices[t].sample < 0 || slices[t].idx_in_sample < 0) return SLIMATTN_ETABLE;
    n_samples = std::max(n_samples, slices[t].sample + 1);
  }
  const int64_t total = (int64_t)3 * n_stages * n_slices;
  *n_buffers = (int32_t)total;
  if (total > cap_buffers) return SLIMATTN_ECAP;
  if (total > 0 && (!buf_stage || !buf_bytes || !buf_alloc_vertex || !buf_free_vertex)) return SLIMATTN_EINVAL;
  // per slice: the first and the last backward unit among the sample's slices at or after it (a sample's slices
  // walked from its last to its first, carrying the running minimum and maximum); per sample: over all slices
  std::vector<std::vector<int32_t>> of_sample(n_samples);
  for (int32_t t = 0; t < n_slices; ++t) of_sample[slices[t].sample].push_back(t);
  std::vector<int32_t> first_b(n_slices), last_b(n_slices), kv_from(n_slices);
  for (auto& ts : of_sample) {
    std::sort(ts.begin(), ts.end(), [&](int32_t a, int32_t b) { return slices[a].idx_in_sample < slices[b].idx_in_sample; });
    int32_t lo = INT32_MAX, hi = -1, f_lo = INT32_MAX;
    for (size_t i = ts.size(); i-- > 0;) {
      lo = std::min(lo, bwd_of[ts[i]]);
      hi = std::max(hi, bwd_of[ts[i]]);
      f_lo = std::min(f_lo, fwd_of[ts[i]]);
      first_b[ts[i]] = lo;
      last_b[ts[i]] = hi;
      kv_from[ts[i]] = fwd_of[ts[i]];
    }
    if (!per_slice)
      for (int32_t t : ts) { first_b[t] = lo; last_b[t] = hi; kv_from[t] = f_lo; }
  }
  auto F = [&](int32_t s, int32_t u) { return s * n_fwd + u; };
  auto B = [&](int32_t s, int32_t v) { return n_stages * n_fwd + s * n_bwd + v; };
  int64_t b = 0;
  auto put = [&](int32_t s, int64_t bytes, int32_t from, int32_t to) {
    buf_stage[b] = s; buf_bytes[b] = bytes; buf_alloc_vertex[b] = from; buf_free_vertex[b] = to;
    ++b;
  };
  for (int32_t s = 0; s < n_stages; ++s)
    for (int32_t t = 0; t < n_slices; ++t) {
      const int64_t n = slices[t].q_len;
      put(s, act_bytes_per_token * n, F(s, fwd_of[t]), B(s, bwd_of[t]));
      put(s, kv_bytes_per_token * n, F(s, kv_from[t]), B(s, last_b[t]));
      put(s, grad_bytes_per_token * n, B(s, first_b[t]), B(s, last_b[t]));
    }
  return SLIMATTN_OK;
}

}  // extern "C"
