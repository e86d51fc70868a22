// Host-side unit-descriptor builder: slice table, grouping policies, validator, cost model.
// Pure host C++ (no HIP).  Integer arithmetic only; the tables it writes are a bit-exact contract.
//
// Paper background: samples are cut into slices and slices are assembled into fixed-budget
// scheduling units with a per-unit target tau = W / m (Two-Phase Objective Formulation, Phase 2);
// the backward pass gets its own partition because attention backward costs 2.5x forward
// (Asymmetric Partition).  The paper solves the assignment with a MILP that it does not print;
// the policies here are deterministic greedy rules of this library's own design.
#include "internal.h"

#include <algorithm>
#include <numeric>
#include <vector>

namespace {

using i128 = __int128;

int64_t pairs_of(const slimattn_slice& s) {
  const int64_t ql = s.q_len, prior = (int64_t)s.kv_len - s.q_len;
  return ql * prior + ql * (ql + 1) / 2;
}

int64_t cost_of(const slimattn_slice& s, int64_t wq, int64_t wl) { return wq * pairs_of(s) + wl * (int64_t)s.q_len; }

// Samples by descending length (ties by index), slices ascending or descending inside a sample.
std::vector<int32_t> walk_order(const int32_t* cu, int32_t n, const slimattn_slice* sl, int32_t ns, bool backward) {
  std::vector<int32_t> first(n + 1, 0);               // counting sort of slice ids by sample
  for (int32_t t = 0; t < ns; ++t) first[sl[t].sample + 1]++;
  for (int32_t s = 0; s < n; ++s) first[s + 1] += first[s];
  std::vector<int32_t> by_sample(ns), fill(first.begin(), first.end() - 1);
  for (int32_t t = 0; t < ns; ++t) by_sample[fill[sl[t].sample]++] = t;   // ascending idx: table order
  std::vector<int32_t> samples(n);
  std::iota(samples.begin(), samples.end(), 0);
  std::stable_sort(samples.begin(), samples.end(), [&](int32_t a, int32_t b) {
    return (cu[a + 1] - cu[a]) > (cu[b + 1] - cu[b]);
  });
  std::vector<int32_t> out;
  out.reserve(ns);
  for (int32_t s : samples) {
    if (backward) for (int32_t i = first[s + 1] - 1; i >= first[s]; --i) out.push_back(by_sample[i]);
    else          for (int32_t i = first[s]; i < first[s + 1]; ++i) out.push_back(by_sample[i]);
  }
  return out;
}

// unit id per position of `seq` by the midpoint rule; ids are non-decreasing along seq.
std::vector<int32_t> midpoint_fill(const std::vector<int32_t>& seq, const slimattn_slice* sl, int32_t m, int64_t wq,
                                   int64_t wl) {
  i128 total = 0;
  for (int32_t t : seq) total += cost_of(sl[t], wq, wl);
  std::vector<int32_t> id(seq.size(), 0);
  i128 before = 0;
  for (size_t i = 0; i < seq.size(); ++i) {
    const i128 c = cost_of(sl[seq[i]], wq, wl);
    i128 u = total > 0 ? ((i128)m * (2 * before + c)) / (2 * total) : 0;
    if (u > m - 1) u = m - 1;
    id[i] = (int32_t)u;
    before += c;
  }
  return id;
}

int emit(const std::vector<std::vector<int32_t>>& groups, int32_t* unit_ptr, int32_t* unit_slices, int32_t cap_units,
         int32_t* n_units) {
  int32_t nu = 0;
  for (auto& g : groups) nu += g.empty() ? 0 : 1;
  *n_units = nu;
  if (nu > cap_units) return SLIMATTN_ECAP;
  int32_t u = 0, pos = 0;
  unit_ptr[0] = 0;
  for (auto& g : groups) {
    if (g.empty()) continue;
    for (int32_t t : g) unit_slices[pos++] = t;
    unit_ptr[++u] = pos;
  }
  return SLIMATTN_OK;
}

}  // namespace

extern "C" {

int64_t slimattn_slice_pairs(const slimattn_slice* s) { return s ? pairs_of(*s) : 0; }
int64_t slimattn_flops_fwd(int64_t pairs, int32_t d, int32_t hq) { return 4 * (int64_t)d * hq * pairs; }
int64_t slimattn_flops_bwd(int64_t pairs, int32_t d, int32_t hq) { return 10 * (int64_t)d * hq * pairs; }

int slimattn_build_slices(const int32_t* lengths, int32_t n, int32_t slice_size, int32_t* cu_out, slimattn_slice* out,
                          int32_t cap, int32_t* n_slices) {
  if (!lengths || !cu_out || !n_slices || n < 0 || slice_size < 1) return SLIMATTN_EINVAL;
  int64_t total = 0, need = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] < 0) return SLIMATTN_EINVAL;
    total += lengths[s];
    need += ((int64_t)lengths[s] + slice_size - 1) / slice_size;
  }
  if (total > INT32_MAX || need > INT32_MAX) return SLIMATTN_EINVAL;
  *n_slices = (int32_t)need;
  cu_out[0] = 0;
  for (int32_t s = 0; s < n; ++s) cu_out[s + 1] = cu_out[s] + lengths[s];
  if (need > cap || (!out && need > 0)) return SLIMATTN_ECAP;
  int32_t t = 0;
  for (int32_t s = 0; s < n; ++s) {
    int32_t idx = 0;
    for (int32_t off = 0; off < lengths[s]; off += slice_size, ++idx, ++t) {
      const int32_t ql = std::min(slice_size, lengths[s] - off);
      out[t] = slimattn_slice{s, idx, cu_out[s] + off, ql, cu_out[s], off + ql, 0, 0};
    }
  }
  return SLIMATTN_OK;
}

int slimattn_build_slices_from_bounds(const int32_t* lengths, int32_t n, const int32_t* bounds_ptr, const int32_t* bounds,
                                      int32_t* cu_out, slimattn_slice* out, int32_t cap, int32_t* n_slices) {
  if (!lengths || !bounds_ptr || !cu_out || !n_slices || n < 0) return SLIMATTN_EINVAL;
  int64_t total = 0, need = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] < 0 || bounds_ptr[s + 1] < bounds_ptr[s]) return SLIMATTN_EINVAL;
    total += lengths[s];
    if (lengths[s] > 0) need += 1 + (bounds_ptr[s + 1] - bounds_ptr[s]);
    int32_t prev = 0;
    for (int32_t i = bounds_ptr[s]; i < bounds_ptr[s + 1]; ++i) {
      if (!bounds || bounds[i] <= prev || bounds[i] >= lengths[s]) return SLIMATTN_EINVAL;
      prev = bounds[i];
    }
  }
  if (total > INT32_MAX) return SLIMATTN_EINVAL;
  *n_slices = (int32_t)need;
  cu_out[0] = 0;
  for (int32_t s = 0; s < n; ++s) cu_out[s + 1] = cu_out[s] + lengths[s];
  if (need > cap || (!out && need > 0)) return SLIMATTN_ECAP;
  int32_t t = 0;
  for (int32_t s = 0; s < n; ++s) {
    if (lengths[s] == 0) continue;
    int32_t a = 0, idx = 0;
    for (int32_t i = bounds_ptr[s]; i <= bounds_ptr[s + 1]; ++i, ++idx, ++t) {
      const int32_t b = (i < bounds_ptr[s + 1]) ? bounds[i] : lengths[s];
      out[t] = slimattn_slice{s, idx, cu_out[s] + a, b - a, cu_out[s], b, 0, 0};
      a = b;
    }
  }
  return SLIMATTN_OK;
}

int slimattn_build_units(const int32_t* cu, int32_t n, const slimattn_slice* sl, int32_t ns, const slimattn_policy* p,
                         int32_t* unit_ptr, int32_t* unit_slices, int32_t cap_units, int32_t* n_units) {
  if (!cu || !p || !unit_ptr || !n_units || n < 0 || ns < 0 || (ns > 0 && (!sl || !unit_slices))) return SLIMATTN_EINVAL;
  for (int32_t t = 0; t < ns; ++t)
    if (sl[t].sample < 0 || sl[t].sample >= n) return SLIMATTN_ETABLE;
  std::vector<std::vector<int32_t>> groups;
  const bool backward = p->backward != 0;
  switch (p->kind) {
    case SLIMATTN_POLICY_ALL: {
      groups.emplace_back(ns);
      std::iota(groups[0].begin(), groups[0].end(), 0);
      break;
    }
    case SLIMATTN_POLICY_PER_SAMPLE: {
      groups.resize(n);
      for (int32_t t = 0; t < ns; ++t) groups[sl[t].sample].push_back(t);
      if (backward) for (auto& g : groups) std::reverse(g.begin(), g.end());
      break;
    }
    case SLIMATTN_POLICY_ROUND_ROBIN: {
      if (p->m < 1) return SLIMATTN_EINVAL;
      groups.resize(p->m);
      for (int32_t t = 0; t < ns; ++t) groups[t % p->m].push_back(t);
      if (p->descending) for (auto& g : groups) std::reverse(g.begin(), g.end());
      break;
    }
    case SLIMATTN_POLICY_PREFIX_FILL: {
      if (p->m < 1) return SLIMATTN_EINVAL;
      const auto seq = walk_order(cu, n, sl, ns, backward);
      const auto id = midpoint_fill(seq, sl, p->m, p->w_quad, p->w_lin);
      groups.resize(p->m);
      for (size_t i = 0; i < seq.size(); ++i) groups[id[i]].push_back(seq[i]);
      break;
    }
    case SLIMATTN_POLICY_TOKEN_CAP: {
      const auto seq = walk_order(cu, n, sl, ns, backward);
      int64_t tokens = 0;
      for (int32_t t : seq) {
        if (groups.empty() || (!groups.back().empty() && tokens + sl[t].q_len > p->cap)) {
          groups.emplace_back();
          tokens = 0;
        }
        groups.back().push_back(t);
        tokens += sl[t].q_len;
      }
      break;
    }
    case SLIMATTN_POLICY_SEEDED_LPT: {
      const auto seq = walk_order(cu, n, sl, ns, backward);
      std::vector<int32_t> per_sample(n, 0);
      for (int32_t t = 0; t < ns; ++t) per_sample[sl[t].sample]++;
      std::vector<i128> load;
      std::vector<int32_t> singles;
      for (int32_t t : seq) {
        if (per_sample[sl[t].sample] > 1) {
          groups.push_back({t});
          load.push_back(cost_of(sl[t], p->w_quad, p->w_lin));
        } else {
          singles.push_back(t);
        }
      }
      while ((int32_t)groups.size() < std::max(1, p->m_min)) { groups.emplace_back(); load.push_back(0); }
      for (int32_t t : singles) {
        size_t best = 0;
        for (size_t u = 1; u < load.size(); ++u) if (load[u] < load[best]) best = u;
        groups[best].push_back(t);
        load[best] += cost_of(sl[t], p->w_quad, p->w_lin);
      }
      break;
    }
    case SLIMATTN_POLICY_ISOLATE_FILL: {
      if (p->m < 1 || p->theta_den < 1 || p->theta_num < 0) return SLIMATTN_EINVAL;
      const auto seq = walk_order(cu, n, sl, ns, backward);
      i128 total = 0;
      for (int32_t t : seq) total += cost_of(sl[t], p->w_quad, p->w_lin);
      std::vector<char> heavy(seq.size(), 0);
      std::vector<int32_t> light;
      int32_t n_heavy = 0;
      for (size_t i = 0; i < seq.size(); ++i) {
        const i128 c = cost_of(sl[seq[i]], p->w_quad, p->w_lin);
        heavy[i] = c * p->m * p->theta_den >= (i128)p->theta_num * total;
        if (heavy[i]) ++n_heavy; else light.push_back(seq[i]);
      }
      const auto id = midpoint_fill(light, sl, std::max(1, p->m - n_heavy), p->w_quad, p->w_lin);
      size_t li = 0;
      int32_t open_id = -1;
      for (size_t i = 0; i < seq.size(); ++i) {
        if (heavy[i]) {
          groups.push_back({seq[i]});
          open_id = -1;
        } else {
          if (id[li] != open_id) { groups.emplace_back(); open_id = id[li]; }
          groups.back().push_back(seq[i]);
          ++li;
        }
      }
      break;
    }
    default:
      return SLIMATTN_EINVAL;
  }
  return emit(groups, unit_ptr, unit_slices, cap_units, n_units);
}

int slimattn_validate(const int32_t* cu, int32_t n, const slimattn_slice* sl, int32_t ns, const int32_t* unit_ptr,
                      const int32_t* unit_slices, int32_t nu, int mode, const char** rule) {
  const char* dummy;
  if (!rule) rule = &dummy;
  *rule = "";
  auto fail = [&](const char* r) { *rule = r; return SLIMATTN_ETABLE; };
  if (!cu || !unit_ptr || n < 0 || ns < 0 || nu < 0 || (ns > 0 && (!sl || !unit_slices))) { *rule = "null"; return SLIMATTN_EINVAL; }
  if (cu[0] != 0) return fail("cu");
  for (int32_t s = 0; s < n; ++s) if (cu[s + 1] < cu[s]) return fail("cu");
  // slices: table order ascending within each sample, exact tiling of [cu[s], cu[s+1])
  std::vector<int32_t> next_row(cu, cu + n), next_idx(n, 0);
  for (int32_t t = 0; t < ns; ++t) {
    const slimattn_slice& x = sl[t];
    if (x.sample < 0 || x.sample >= n) return fail("sample_range");
    if (x.idx_in_sample != next_idx[x.sample] || x.q_start != next_row[x.sample] || x.q_len <= 0) return fail("tiling");
    if ((int64_t)x.q_start + x.q_len > cu[x.sample + 1]) return fail("tiling");
    if (x.kv_start != cu[x.sample] || x.kv_len != x.q_start + x.q_len - cu[x.sample]) return fail("kv_range");
    next_row[x.sample] += x.q_len;
    next_idx[x.sample]++;
  }
  for (int32_t s = 0; s < n; ++s) if (next_row[s] != cu[s + 1]) return fail("tiling");
  if (unit_ptr[0] != 0) return fail("unit_ptr");
  for (int32_t u = 0; u < nu; ++u) if (unit_ptr[u + 1] < unit_ptr[u]) return fail("unit_ptr");
  if (unit_ptr[nu] != ns) return fail("coverage");
  std::vector<int32_t> unit_of(ns, -1), pos_of(ns, -1);
  for (int32_t u = 0; u < nu; ++u)
    for (int32_t i = unit_ptr[u]; i < unit_ptr[u + 1]; ++i) {
      const int32_t t = unit_slices[i];
      if (t < 0 || t >= ns) return fail("slice_range");
      if (unit_of[t] != -1) return fail("coverage");
      unit_of[t] = u;
      pos_of[t] = i;
    }
  if (mode & SLIMATTN_CHECK_ORDER) {
    const bool backward = (mode & SLIMATTN_CHECK_BACKWARD) != 0;
    std::vector<int32_t> prev(n, -1);                  // previous slice (lower idx) of each sample
    for (int32_t t = 0; t < ns; ++t) {
      const int32_t a = prev[sl[t].sample];
      prev[sl[t].sample] = t;
      if (a < 0) continue;
      if (backward ? unit_of[a] < unit_of[t] : unit_of[a] > unit_of[t]) return fail("unit_order");
      if (unit_of[a] == unit_of[t] && pos_of[t] - pos_of[a] != (backward ? -1 : 1)) return fail("adjacency");
    }
  }
  return SLIMATTN_OK;
}

const char* slimattn_strerror(int code) {
  switch (code) {
    case SLIMATTN_OK: return "ok";
    case SLIMATTN_EINVAL: return "invalid argument";
    case SLIMATTN_ETABLE: return "inconsistent tables";
    case SLIMATTN_ECAP: return "output capacity too small";
    case SLIMATTN_EHIP: return "HIP call failed";
    case SLIMATTN_ENOMEM: return "out of host memory";
    case SLIMATTN_EINFEASIBLE: return "the token cap needs more units than allowed";
    case SLIMATTN_ESCRATCH: return "workspace need exceeds the built-in scratch array";
    default: return "unknown error";
  }
}

int slimattn_version(void) { return 100; }

}  // extern "C"
