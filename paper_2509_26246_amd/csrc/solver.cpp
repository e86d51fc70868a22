// Partition solver: exact min-max cut of the packed samples into at most m scheduling units per pass, slice
// boundaries included.  Pure host C++, integer arithmetic only.
//
// Paper background (Balanced Packing & Asymmetric Partitioning Solver): Phase 2 gives every unit the target
// tau = W / m, cuts long samples into slices spread over several units and packs short samples together, and
// the slice boundaries are an output of the optimisation; the Asymmetric Partition paragraph asks for a second
// partition of the same samples computed from backward costs (attention backward costs 2.5 x forward), in the
// same unit order; the candidate search evaluates several unit counts m.  The paper's MILP is not printed.
// Here the problem is stated so that it has an exact, fast solution: a unit is a contiguous piece of the walk
// (samples by descending length; rows upwards in the forward pass, downwards in the backward pass), a row that
// sees i + 1 keys costs w_quad * (i + 1) + w_lin, cuts fall on multiples of `granule` rows from a sample's
// start.  Costs are additive over rows, so "at most m contiguous parts with the smallest largest part" is
// solved by a search over the bound B with a greedy feasibility test (close a unit when the next granule
// would exceed B or the token cap), which is optimal for additive costs.  The cuts reported are the greedy
// ones at the optimal bound.  The slice table is the union of both passes' cuts.
#include "internal.h"

#include <algorithm>
#include <atomic>
#include <numeric>
#include <thread>
#include <vector>

namespace {

struct Granule { int32_t sample, a, b; int64_t cost; };

int64_t rows_cost(int64_t a, int64_t b, int64_t wq, int64_t wl) {
  const int64_t n = b - a;
  return wq * (n * a + n * (n + 1) / 2) + wl * n;
}

std::vector<int32_t> sample_order(const int32_t* lengths, int32_t n) {
  std::vector<int32_t> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return lengths[x] > lengths[y]; });
  return order;
}

std::vector<Granule> walk(const int32_t* lengths, const std::vector<int32_t>& order, int32_t granule, int64_t wq, int64_t wl,
                          bool backward) {
  std::vector<Granule> out;
  for (int32_t s : order) {
    const int32_t L = lengths[s];
    const size_t first = out.size();
    for (int32_t a = 0; a < L; a += granule) {
      const int32_t b = std::min(L, a + granule);
      out.push_back(Granule{s, a, b, rows_cost(a, b, wq, wl)});
    }
    if (backward) std::reverse(out.begin() + first, out.end());
  }
  return out;
}

// Units the greedy rule needs under bound B; `starts` (optional) receives each unit's first granule.
int64_t greedy_units(const std::vector<Granule>& gr, int64_t B, int64_t cap, std::vector<int32_t>* starts) {
  int64_t units = 0, c = 0, t = 0;
  for (size_t i = 0; i < gr.size(); ++i) {
    const int64_t ti = gr[i].b - gr[i].a;
    if (i == 0 || c + gr[i].cost > B || (cap > 0 && t + ti > cap)) {
      ++units;
      if (starts) starts->push_back((int32_t)i);
      c = 0;
      t = 0;
    }
    c += gr[i].cost;
    t += ti;
  }
  return units;
}

// Smallest bound under which at most m units suffice; -1 if the token cap alone forces more than m units.
int64_t bottleneck(const std::vector<Granule>& gr, int32_t m, int64_t cap) {
  if (gr.empty()) return 0;
  int64_t lo = 0, hi = 0;
  for (const Granule& g : gr) { lo = std::max(lo, g.cost); hi += g.cost; }
  if (greedy_units(gr, hi, cap, nullptr) > m) return -1;
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (greedy_units(gr, mid, cap, nullptr) <= m) hi = mid; else lo = mid + 1;
  }
  return lo;
}

bool params_ok(const slimattn_solver* sp) {
  return sp && sp->m_fwd >= 1 && sp->m_bwd >= 1 && sp->granule >= 1 && sp->w_quad_fwd >= 0 && sp->w_lin_fwd >= 0 &&
         sp->w_quad_bwd >= 0 && sp->w_lin_bwd >= 0 && sp->token_cap_fwd >= 0 && sp->token_cap_bwd >= 0 && sp->max_slice >= 0 &&
         sp->w_quad_fwd <= (int64_t(1) << 20) && sp->w_quad_bwd <= (int64_t(1) << 20) && sp->w_lin_fwd <= (int64_t(1) << 30) &&
         sp->w_lin_bwd <= (int64_t(1) << 30);
}

bool lengths_ok(const int32_t* lengths, int32_t n) {
  int64_t total = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] < 0) return false;
    total += lengths[s];
  }
  return total <= INT32_MAX / 2;      // costs then stay far inside 64 bits: 2^20 * 2^59 is out of reach with T < 2^30
}

}  // namespace

extern "C" {

int slimattn_solve_partition(const int32_t* lengths, int32_t n, const slimattn_solver* sp, int32_t* cu_out,
                             slimattn_slice* slices, int32_t cap_slices, int32_t* n_slices, int32_t* fwd_unit_ptr,
                             int32_t* fwd_unit_slices, int32_t* n_fwd_units, int32_t* bwd_unit_ptr, int32_t* bwd_unit_slices,
                             int32_t* n_bwd_units, int32_t cap_units, int64_t* bottlenecks) {
  if (!lengths || n < 0 || !params_ok(sp) || !cu_out || !n_slices || !n_fwd_units || !n_bwd_units || !fwd_unit_ptr || !bwd_unit_ptr)
    return SLIMATTN_EINVAL;
  if (!lengths_ok(lengths, n)) return SLIMATTN_EINVAL;
  const std::vector<int32_t> order = sample_order(lengths, n);
  cu_out[0] = 0;
  for (int32_t s = 0; s < n; ++s) cu_out[s + 1] = cu_out[s] + lengths[s];

  // both passes: bound, greedy cuts, each unit's row range per sample
  struct Piece { int32_t sample, lo, hi; };                    // a unit holds one contiguous row range of a sample
  std::vector<std::vector<Piece>> units[2];
  std::vector<std::vector<int32_t>> cuts(n);
  for (int pass = 0; pass < 2; ++pass) {
    const bool backward = pass == 1;
    const std::vector<Granule> gr = walk(lengths, order, sp->granule, backward ? sp->w_quad_bwd : sp->w_quad_fwd,
                                         backward ? sp->w_lin_bwd : sp->w_lin_fwd, backward);
    const int64_t cap = backward ? sp->token_cap_bwd : sp->token_cap_fwd;
    const int64_t B = bottleneck(gr, backward ? sp->m_bwd : sp->m_fwd, cap);
    if (B < 0) return SLIMATTN_EINFEASIBLE;
    if (bottlenecks) bottlenecks[pass] = B;
    std::vector<int32_t> starts;
    greedy_units(gr, B, cap, &starts);
    starts.push_back((int32_t)gr.size());
    for (size_t u = 0; u + 1 < starts.size(); ++u) {
      std::vector<Piece> pieces;
      for (int32_t i = starts[u]; i < starts[u + 1]; ++i) {
        if (!pieces.empty() && pieces.back().sample == gr[i].sample) {
          pieces.back().lo = std::min(pieces.back().lo, gr[i].a);
          pieces.back().hi = std::max(pieces.back().hi, gr[i].b);
        } else {
          pieces.push_back(Piece{gr[i].sample, gr[i].a, gr[i].b});
        }
      }
      for (const Piece& p : pieces) {
        if (p.lo > 0) cuts[p.sample].push_back(p.lo);
        if (p.hi < lengths[p.sample]) cuts[p.sample].push_back(p.hi);
      }
      units[pass].push_back(std::move(pieces));
    }
  }
  if (sp->max_slice > 0)
    for (int32_t s = 0; s < n; ++s)
      for (int32_t c = sp->max_slice; c < lengths[s]; c += sp->max_slice) cuts[s].push_back(c);

  // slice table: samples in index order, slices ascending
  std::vector<int32_t> first_slice(n + 1, 0);
  int64_t need = 0;
  for (int32_t s = 0; s < n; ++s) {
    std::sort(cuts[s].begin(), cuts[s].end());
    cuts[s].erase(std::unique(cuts[s].begin(), cuts[s].end()), cuts[s].end());
    first_slice[s] = (int32_t)need;
    if (lengths[s] > 0) need += 1 + (int64_t)cuts[s].size();
  }
  first_slice[n] = (int32_t)need;
  *n_slices = (int32_t)need;
  *n_fwd_units = (int32_t)units[0].size();
  *n_bwd_units = (int32_t)units[1].size();
  if (need > cap_slices || (int64_t)std::max(units[0].size(), units[1].size()) > cap_units) return SLIMATTN_ECAP;
  if (need > 0 && (!slices || !fwd_unit_slices || !bwd_unit_slices)) return SLIMATTN_EINVAL;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] == 0) continue;
    int32_t a = 0, idx = 0, t = first_slice[s];
    for (size_t i = 0; i <= cuts[s].size(); ++i, ++idx, ++t) {
      const int32_t b = i < cuts[s].size() ? cuts[s][i] : lengths[s];
      slices[t] = slimattn_slice{s, idx, cu_out[s] + a, b - a, cu_out[s], b, 0, 0};
      a = b;
    }
  }
  // unit lists: the slices inside each unit's row ranges, in walk order
  for (int pass = 0; pass < 2; ++pass) {
    int32_t* ptr = pass ? bwd_unit_ptr : fwd_unit_ptr;
    int32_t* flat = pass ? bwd_unit_slices : fwd_unit_slices;
    int32_t pos = 0;
    ptr[0] = 0;
    for (size_t u = 0; u < units[pass].size(); ++u) {
      for (const Piece& p : units[pass][u]) {
        // slices of the sample with start row in [p.lo, p.hi): a contiguous run of table indices
        const std::vector<int32_t>& c = cuts[p.sample];
        const int32_t i0 = p.lo == 0 ? 0 : (int32_t)(std::lower_bound(c.begin(), c.end(), p.lo) - c.begin()) + 1;
        const int32_t i1 = p.hi == lengths[p.sample] ? (int32_t)c.size() + 1 : (int32_t)(std::lower_bound(c.begin(), c.end(), p.hi) - c.begin()) + 1;
        if (pass == 0) for (int32_t i = i0; i < i1; ++i) flat[pos++] = first_slice[p.sample] + i;
        else for (int32_t i = i1 - 1; i >= i0; --i) flat[pos++] = first_slice[p.sample] + i;
      }
      ptr[u + 1] = pos;
    }
  }
  return SLIMATTN_OK;
}

int slimattn_solve_bottlenecks(const int32_t* lengths, int32_t n, const slimattn_solver* sp, const int32_t* m_list, int32_t n_m,
                               int32_t n_threads, int64_t* fwd_bottleneck, int64_t* bwd_bottleneck) {
  if (!lengths || n < 0 || !params_ok(sp) || n_m < 0 || (n_m > 0 && (!m_list || !fwd_bottleneck || !bwd_bottleneck)))
    return SLIMATTN_EINVAL;
  if (!lengths_ok(lengths, n)) return SLIMATTN_EINVAL;
  for (int32_t i = 0; i < n_m; ++i)
    if (m_list[i] < 1) return SLIMATTN_EINVAL;
  const std::vector<int32_t> order = sample_order(lengths, n);
  const std::vector<Granule> gf = walk(lengths, order, sp->granule, sp->w_quad_fwd, sp->w_lin_fwd, false);
  const std::vector<Granule> gb = walk(lengths, order, sp->granule, sp->w_quad_bwd, sp->w_lin_bwd, true);
  // a small pool: workers take the next (candidate, pass) job from a shared counter
  std::atomic<int32_t> next{0};
  auto work = [&]() {
    for (int32_t job = next.fetch_add(1); job < 2 * n_m; job = next.fetch_add(1)) {
      const int32_t i = job / 2;
      if (job % 2 == 0) fwd_bottleneck[i] = bottleneck(gf, m_list[i], sp->token_cap_fwd);
      else bwd_bottleneck[i] = bottleneck(gb, m_list[i], sp->token_cap_bwd);
    }
  };
  const int32_t workers = std::max(1, std::min<int32_t>(std::min(n_threads, 64), 2 * n_m));
  std::vector<std::thread> pool;
  try {
    for (int32_t w = 1; w < workers; ++w) pool.emplace_back(work);
  } catch (...) {
    // fewer threads than asked for: the calling thread does the rest
  }
  work();
  for (std::thread& th : pool) th.join();
  return SLIMATTN_OK;
}

}  // extern "C"
