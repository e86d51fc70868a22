// Search over the number of scheduling units: for each candidate m the partition solver's units go through the
// pipeline simulator, and the candidate with the shortest simulated iteration that fits the memory limit wins.
// Pure host C++, integers only.
//
// Paper: Balanced Packing & Asymmetric Partitioning Solver (the number of MicroPacks m sets the per-unit budget
// W / m; several m are evaluated); Primitive Measurements and Search Space (m is taken from multiples of the
// pipeline width on a roughly logarithmic grid; runtimes are estimated from FLOPs with utilisations calibrated
// by preliminary benchmarks); DAG-based Pipeline Simulator (execution time and memory footprint of a candidate).
// A task's time is fixed + cost * num / den (integer division), cost = w_quad * pairs + w_lin * rows of its
// slices with the pass's weights: the fixed part is the per-launch overhead the calibration measures, the rest
// the calibrated rate.
#include "internal.h"

#include <algorithm>
#include <atomic>
#include <thread>
#include <vector>

namespace {

bool rate_ok(int64_t fixed, int64_t num, int64_t den) { return fixed >= 0 && num >= 0 && den >= 1 && num <= (int64_t(1) << 31); }

// One candidate: simulated iteration time and the worst stage's peak; rc != OK on errors, *t_total = -1 if the
// token cap makes m units infeasible.
int evaluate(const int32_t* lengths, int32_t n, const slimattn_solver& base, const slimattn_search& ss, int32_t m,
             int64_t* t_total, int64_t* peak) {
  slimattn_solver sp = base;
  sp.m_fwd = m;
  sp.m_bwd = m;
  int64_t total = 0;
  for (int32_t s = 0; s < n; ++s) total += lengths[s];
  // every granule could become a slice of its own, and max_slice adds at most total / max_slice + n more
  const int64_t cap_slices64 = total / sp.granule + 2 * (int64_t)n + (sp.max_slice > 0 ? total / sp.max_slice + n : 0) + 4 * (int64_t)m + 8;
  const int32_t cap_slices = (int32_t)std::min<int64_t>(cap_slices64, INT32_MAX / 2);
  std::vector<int32_t> cu(n + 1), fp(m + 2), fs(cap_slices), bp(m + 2), bs(cap_slices);
  std::vector<slimattn_slice> sl(cap_slices);
  int32_t n_sl = 0, nf = 0, nb = 0;
  int rc = slimattn_solve_partition(lengths, n, &sp, cu.data(), sl.data(), cap_slices, &n_sl, fp.data(), fs.data(), &nf, bp.data(),
                                    bs.data(), &nb, m + 1, nullptr);
  if (rc == SLIMATTN_EINFEASIBLE) { *t_total = -1; *peak = -1; return SLIMATTN_OK; }
  if (rc != SLIMATTN_OK) return rc;
  auto unit_time = [&](const int32_t* ptr, const int32_t* flat, int32_t u, int64_t wq, int64_t wl, int64_t fixed, int64_t num, int64_t den) {
    int64_t cost = 0;
    for (int32_t i = ptr[u]; i < ptr[u + 1]; ++i) cost += wq * slimattn_slice_pairs(&sl[flat[i]]) + wl * sl[flat[i]].q_len;
    return fixed + (int64_t)((__int128)cost * num / den);
  };
  std::vector<int64_t> fc(nf), bc(nb);
  for (int32_t u = 0; u < nf; ++u) fc[u] = unit_time(fp.data(), fs.data(), u, sp.w_quad_fwd, sp.w_lin_fwd, ss.fwd_fixed, ss.fwd_num, ss.fwd_den);
  for (int32_t u = 0; u < nb; ++u) bc[u] = unit_time(bp.data(), bs.data(), u, sp.w_quad_bwd, sp.w_lin_bwd, ss.bwd_fixed, ss.bwd_num, ss.bwd_den);
  const int32_t p = ss.n_stages;
  const int64_t nv64 = (int64_t)p * (nf + nb);
  if (nv64 > INT32_MAX / 8) return SLIMATTN_EINVAL;
  int32_t nv = 0, ne = 0;
  rc = slimattn_dag_build_1f1b(sl.data(), n_sl, fp.data(), fs.data(), nf, bp.data(), bs.data(), nb, p, fc.data(), bc.data(), nullptr, nullptr, 0,
                               &nv, nullptr, nullptr, nullptr, 0, &ne);
  if (rc != SLIMATTN_OK && rc != SLIMATTN_ECAP) return rc;
  std::vector<int32_t> vertex(3 * (size_t)std::max(nv, 1)), ef(std::max(ne, 1)), et(std::max(ne, 1)), ek(std::max(ne, 1));
  std::vector<int64_t> weight(std::max(nv, 1)), start(std::max(nv, 1)), finish(std::max(nv, 1));
  rc = slimattn_dag_build_1f1b(sl.data(), n_sl, fp.data(), fs.data(), nf, bp.data(), bs.data(), nb, p, fc.data(), bc.data(), vertex.data(),
                               weight.data(), nv, &nv, ef.data(), et.data(), ek.data(), ne, &ne);
  if (rc != SLIMATTN_OK) return rc;
  rc = slimattn_dag_timeline(nv, weight.data(), ne, ef.data(), et.data(), start.data(), finish.data(), t_total);
  if (rc != SLIMATTN_OK) return rc;
  const int32_t n_buf = 3 * p * n_sl;
  std::vector<int32_t> b_stage(std::max(n_buf, 1)), b_alloc(std::max(n_buf, 1)), b_free(std::max(n_buf, 1));
  std::vector<int64_t> b_bytes(std::max(n_buf, 1)), pk(p), pt(p);
  int32_t got = 0;
  rc = slimattn_dag_buffers_1f1b(sl.data(), n_sl, fp.data(), fs.data(), nf, bp.data(), bs.data(), nb, p, ss.act_bytes_per_token,
                                 ss.kv_bytes_per_token, ss.grad_bytes_per_token, 1, b_stage.data(), b_bytes.data(), b_alloc.data(),
                                 b_free.data(), n_buf, &got);
  if (rc != SLIMATTN_OK) return rc;
  rc = slimattn_dag_memory(nv, start.data(), finish.data(), got, b_stage.data(), b_bytes.data(), b_alloc.data(), b_free.data(), p, nullptr,
                           pk.data(), pt.data());
  if (rc != SLIMATTN_OK) return rc;
  *peak = *std::max_element(pk.begin(), pk.end());
  return SLIMATTN_OK;
}

}  // namespace

extern "C" {

int slimattn_candidate_unit_counts(int32_t n_stages, int32_t m_max, int32_t* out, int32_t cap, int32_t* n_out) {
  if (n_stages < 1 || m_max < 0 || cap < 0 || !n_out || (cap > 0 && !out)) return SLIMATTN_EINVAL;
  // i = 1, 2, 3, 4, 6, 8, 12, 16, 24, ...: the powers of two and the values halfway between them
  int32_t count = 0;
  for (int64_t pow2 = 1;; pow2 *= 2) {
    const int64_t pair[2] = {pow2, pow2 >= 2 ? pow2 + pow2 / 2 : 0};
    bool any = false;
    for (int64_t i : pair) {
      if (i == 0 || i * n_stages > m_max) continue;
      any = true;
      if (count < cap) out[count] = (int32_t)(i * n_stages);
      ++count;
    }
    if (!any) break;
  }
  *n_out = count;
  return count > cap ? SLIMATTN_ECAP : SLIMATTN_OK;
}

int slimattn_search_unit_count(const int32_t* lengths, int32_t n, const slimattn_solver* sp, const slimattn_search* ss,
                               const int32_t* m_list, int32_t n_m, int32_t n_threads, int64_t* t_total, int64_t* peak_bytes,
                               int32_t* best) {
  if (!lengths || n < 0 || !sp || !ss || n_m < 0 || !best || (n_m > 0 && (!m_list || !t_total || !peak_bytes))) return SLIMATTN_EINVAL;
  if (ss->n_stages < 1 || !rate_ok(ss->fwd_fixed, ss->fwd_num, ss->fwd_den) || !rate_ok(ss->bwd_fixed, ss->bwd_num, ss->bwd_den) ||
      ss->act_bytes_per_token < 0 || ss->kv_bytes_per_token < 0 || ss->grad_bytes_per_token < 0 || ss->stage_bytes_cap < 0)
    return SLIMATTN_EINVAL;
  for (int32_t i = 0; i < n_m; ++i)
    if (m_list[i] < 1) return SLIMATTN_EINVAL;
  std::vector<int> rcs(n_m, SLIMATTN_OK);
  std::atomic<int32_t> next{0};
  auto work = [&]() {
    for (int32_t i = next.fetch_add(1); i < n_m; i = next.fetch_add(1)) rcs[i] = evaluate(lengths, n, *sp, *ss, m_list[i], &t_total[i], &peak_bytes[i]);
  };
  const int32_t workers = std::max(1, std::min<int32_t>(std::min(n_threads, 64), n_m));
  std::vector<std::thread> pool;
  try {
    for (int32_t w = 1; w < workers; ++w) pool.emplace_back(work);
  } catch (...) {
    // fewer threads than asked for: the calling thread does the rest
  }
  work();
  for (std::thread& th : pool) th.join();
  for (int32_t i = 0; i < n_m; ++i)
    if (rcs[i] != SLIMATTN_OK) return rcs[i];
  *best = -1;
  for (int32_t i = 0; i < n_m; ++i) {
    if (t_total[i] < 0 || (ss->stage_bytes_cap > 0 && peak_bytes[i] > ss->stage_bytes_cap)) continue;
    if (*best < 0 || t_total[i] < t_total[*best]) *best = i;      // ties: the earlier entry of the list
  }
  return SLIMATTN_OK;
}

}  // extern "C"
