// Table handle: validation, derived tile work-lists, device upload.
//
// The derived lists are private to the library.  A launch scope is one unit, or the whole list.
// Inside a scope the slices of a sample that touch each other are merged into runs of query rows;
// runs are cut into query tiles (forward, dQ) and the sample prefix they can see is cut into key
// tiles (dK/dV: the tile's owner sums the contributions of every run that ends after it: a slice's
// key/value gradients are complete only once every later slice of its sample has run -- the
// inter-slice dependency of the backward pass in the paper's DAG simulator section).  Items are
// ordered heavy-first so that the hardware's in-order block dispatch acts as a
// longest-processing-time schedule.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>

#include "internal.h"

namespace slimattn {
namespace {

thread_local int g_last_hip_error = 0;

// Runs of one scope: slices (any order) -> per sample, ascending, adjacent slices merged.
struct Run { int32_t sample, q_lo, q_hi, kv_start; };

std::vector<Run> merge_runs(const slimattn_slice* sl, const int32_t* ids, int32_t count) {
  std::vector<Run> runs;
  runs.reserve(count);
  for (int32_t i = 0; i < count; ++i) {
    const slimattn_slice& s = sl[ids[i]];
    runs.push_back(Run{s.sample, s.q_start, s.q_start + s.q_len, s.kv_start});
  }
  std::sort(runs.begin(), runs.end(), [](const Run& a, const Run& b) { return a.q_lo < b.q_lo; });
  std::vector<Run> out;
  for (const Run& r : runs) {
    if (!out.empty() && out.back().sample == r.sample && out.back().q_hi == r.q_lo) out.back().q_hi = r.q_hi;
    else out.push_back(r);
  }
  return out;
}

// Divided variants of one scope's 256-row key tiles.  With h KV heads a launch has items x h
// blocks on kBlockSlots resident slots, so a tile whose query rows exceed a fraction of the
// per-slot share W * h / kBlockSlots is cut into parts of about half a share (parts no shorter
// than kMinPartRows).  A part is an item of
// its own, with its own (cut) runs appended to segs and a partial-tile slot; slots of one tile are
// consecutive and the reduction adds them in that order, so results do not depend on scheduling.
constexpr int64_t kMinPartRows = 256;

void append_split(ScopeLists& L, int ti, const std::vector<KvItem>& ki, const std::vector<int64_t>& weight) {
  const int64_t kBlockSlots = kSplitBlockSlots[ti];
  int64_t total = 0;
  for (int64_t w : weight) total += w;
  for (int c = 0; c < kNumSplitClasses; ++c) {
    const int64_t heads = int64_t(1) << c;
    // A tile is divided when it exceeds three quarters of the per-slot share (below that, the
    // heavy-first dispatch already hides it), into parts of about half a share: the divided tiles
    // then no longer decide the makespan.
    const int64_t share = total * heads / kBlockSlots;
    const int64_t target = std::max(kMinPartRows, (share / 2 + 127) / 128 * 128);
    std::vector<KvItem> items;
    std::vector<int64_t> w;
    int32_t slots = 0;
    for (size_t x = 0; x < ki.size(); ++x) {
      const int64_t parts = std::min<int64_t>((weight[x] + target - 1) / target, weight[x] / kMinPartRows);
      if (parts < 2 || 4 * weight[x] <= 3 * share) {
        items.push_back(ki[x]);
        w.push_back(weight[x]);
        continue;
      }
      const int64_t chunk = ((weight[x] + parts - 1) / parts + 127) / 128 * 128;
      L.reduce_items[ti][c].push_back(KvReduce{ki[x].kv_row0, ki[x].kv_rows, slots, 0, ki[x].load_until, ki[x].final_from, 0, 0});
      KvReduce& red = L.reduce_items[ti][c].back();
      // walk the tile's runs, closing a part whenever it holds `chunk` rows
      int64_t have = 0;
      int32_t part_seg_begin = (int32_t)L.segs.size();
      auto close_part = [&]() {
        items.push_back(KvItem{ki[x].kv_row0, ki[x].kv_rows, part_seg_begin, (int32_t)L.segs.size(), slots, 0, 0, 0});
        w.push_back(have);
        ++slots;
        ++red.n_parts;
        have = 0;
        part_seg_begin = (int32_t)L.segs.size();
      };
      for (int32_t sgi = ki[x].seg_begin; sgi < ki[x].seg_end; ++sgi) {
        const Seg sg = L.segs[sgi];
        int32_t a = std::max(sg.q_lo, ki[x].kv_row0);
        while (a < sg.q_hi) {
          const int32_t take = (int32_t)std::min<int64_t>(sg.q_hi - a, chunk - have);
          L.segs.push_back(Seg{a, a + take});
          have += take;
          a += take;
          if (have == chunk) close_part();
        }
      }
      if (have > 0) close_part();
    }
    std::vector<int32_t> order(items.size());
    for (size_t x = 0; x < order.size(); ++x) order[x] = (int32_t)x;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return w[a] > w[b]; });
    for (int32_t x : order) L.split_items[ti][c].push_back(items[x]);
    L.split_off[ti][c].push_back((int32_t)L.split_items[ti][c].size());
    L.reduce_off[ti][c].push_back((int32_t)L.reduce_items[ti][c].size());
    L.max_slots[ti][c] = std::max(L.max_slots[ti][c], slots);
  }
}

// `row_marks(sample)`: {load_until, final_from} of the sample's key rows for this scope.
// want_kv: key-tile lists are only needed by the backward pass.
template <class Marks>
void append_scope(ScopeLists& L, const std::vector<Run>& runs, bool want_kv, Marks&& row_marks) {
  const int32_t seg_base = (int32_t)L.segs.size();
  for (const Run& r : runs) L.segs.push_back(Seg{r.q_lo, r.q_hi});
  for (int z = 0; z < kNumTileSizes; ++z) {
    const int32_t B = kTileSizes[z];
    // query tiles, heavy-first by visible prefix length
    std::vector<QItem> qi;
    if (is_query_tile(B))
      for (const Run& r : runs)
        for (int32_t a = r.q_lo; a < r.q_hi; a += B) qi.push_back(QItem{a, std::min(B, r.q_hi - a), r.kv_start, 0});
    std::stable_sort(qi.begin(), qi.end(), [](const QItem& a, const QItem& b) {
      return (a.q_row0 + a.q_rows - a.kv_start) > (b.q_row0 + b.q_rows - b.kv_start);
    });
    L.q_items[z].insert(L.q_items[z].end(), qi.begin(), qi.end());
    L.q_off[z].push_back((int32_t)L.q_items[z].size());
    // key tiles: per sample, prefix [kv_start, last run's end); heavy-first by query rows at or after the tile
    std::vector<KvItem> ki;
    std::vector<int64_t> weight;
    size_t i = (want_kv && is_key_tile(B)) ? 0 : runs.size();
    while (i < runs.size()) {
      size_t j = i;
      while (j < runs.size() && runs[j].sample == runs[i].sample) ++j;
      const int32_t kv0 = runs[i].kv_start, kv_end = runs[j - 1].q_hi;
      const std::pair<int32_t, int32_t> marks = row_marks(runs[i].sample);
      for (int32_t a = kv0; a < kv_end; a += B) {
        size_t first = i;
        while (runs[first].q_hi <= a) ++first;             // exists: the last run ends after a
        int64_t rows = 0;
        for (size_t r = first; r < j; ++r) rows += runs[r].q_hi - std::max(runs[r].q_lo, a);
        ki.push_back(KvItem{a, std::min(B, kv_end - a), seg_base + (int32_t)first, seg_base + (int32_t)j, -1,
                            marks.first, marks.second, 0});
        weight.push_back(rows);
      }
      i = j;
    }
    std::vector<int32_t> order(ki.size());
    for (size_t x = 0; x < order.size(); ++x) order[x] = (int32_t)x;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return weight[a] > weight[b]; });
    for (int32_t x : order) L.kv_items[z].push_back(ki[x]);
    L.kv_off[z].push_back((int32_t)L.kv_items[z].size());
    if (split_tile_index(B) >= 0) append_split(L, split_tile_index(B), ki, weight);
  }
}

size_t align_up(size_t x) { return (x + 255) & ~size_t(255); }

template <class T>
size_t place(std::vector<char>& blob, const std::vector<T>& v) {
  const size_t off = align_up(blob.size());
  blob.resize(off + v.size() * sizeof(T));
  if (!v.empty()) std::memcpy(blob.data() + off, v.data(), v.size() * sizeof(T));
  return off;
}

}  // namespace

int& last_hip_error() { return g_last_hip_error; }

}  // namespace slimattn

using namespace slimattn;

extern "C" {

int slimattn_last_hip_error(void) { return g_last_hip_error; }

int slimattn_tables_create(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                           const int32_t* fwd_unit_ptr, const int32_t* fwd_unit_slices, int32_t n_fwd_units,
                           const int32_t* bwd_unit_ptr, const int32_t* bwd_unit_slices, int32_t n_bwd_units,
                           slimattn_tables** out) {
  return slimattn_tables_create_async(cu, n, slices, n_slices, fwd_unit_ptr, fwd_unit_slices, n_fwd_units, bwd_unit_ptr,
                                      bwd_unit_slices, n_bwd_units, nullptr, 0, out);
}

int slimattn_tables_create_async(const int32_t* cu, int32_t n, const slimattn_slice* slices, int32_t n_slices,
                                 const int32_t* fwd_unit_ptr, const int32_t* fwd_unit_slices, int32_t n_fwd_units,
                                 const int32_t* bwd_unit_ptr, const int32_t* bwd_unit_slices, int32_t n_bwd_units,
                                 void* stream, int use_stream, slimattn_tables** out) {
  if (!out) return SLIMATTN_EINVAL;
  *out = nullptr;
  int rc = slimattn_validate(cu, n, slices, n_slices, fwd_unit_ptr, fwd_unit_slices, n_fwd_units, SLIMATTN_CHECK_FORWARD, nullptr);
  if (rc != SLIMATTN_OK) return rc;
  rc = slimattn_validate(cu, n, slices, n_slices, bwd_unit_ptr, bwd_unit_slices, n_bwd_units, SLIMATTN_CHECK_BACKWARD, nullptr);
  if (rc != SLIMATTN_OK) return rc;
  slimattn_tables* t = new (std::nothrow) slimattn_tables();
  if (!t) return SLIMATTN_ENOMEM;
  try {
    t->n_samples = n;
    t->n_slices = n_slices;
    t->n_units[0] = n_fwd_units;
    t->n_units[1] = n_bwd_units;
    t->total_tokens = cu[n];
    for (int32_t i = 0; i < n; ++i) t->max_sample_len = std::max(t->max_sample_len, cu[i + 1] - cu[i]);
    t->cu.assign(cu, cu + n + 1);
    t->slices.assign(slices, slices + n_slices);
    t->unit_ptr[0].assign(fwd_unit_ptr, fwd_unit_ptr + n_fwd_units + 1);
    t->unit_slices[0].assign(fwd_unit_slices, fwd_unit_slices + n_slices);
    t->unit_ptr[1].assign(bwd_unit_ptr, bwd_unit_ptr + n_bwd_units + 1);
    t->unit_slices[1].assign(bwd_unit_slices, bwd_unit_slices + n_slices);
    for (int pass = 0; pass < 2; ++pass) {
      for (int z = 0; z < kNumTileSizes; ++z) { t->per_unit[pass].q_off[z].push_back(0); t->per_unit[pass].kv_off[z].push_back(0); }
      for (int ti = 0; ti < kNumSplitTiles; ++ti)
        for (int c = 0; c < kNumSplitClasses; ++c) { t->per_unit[pass].split_off[ti][c].push_back(0); t->per_unit[pass].reduce_off[ti][c].push_back(0); }
      // reach[s]: (unit, end of the unit's last query row in sample s), in list order.  A unit collects into the
      // key tiles of the sample that start before that end.
      std::vector<std::vector<std::pair<int32_t, int32_t>>> reach(n);
      for (int32_t u = 0; u < t->n_units[pass]; ++u)
        for (int32_t i = t->unit_ptr[pass][u]; i < t->unit_ptr[pass][u + 1]; ++i) {
          const slimattn_slice& x = slices[t->unit_slices[pass][i]];
          auto& r = reach[x.sample];
          if (!r.empty() && r.back().first == u) r.back().second = std::max(r.back().second, x.q_start + x.q_len);
          else r.emplace_back(u, x.q_start + x.q_len);
        }
      for (int32_t u = 0; u < t->n_units[pass]; ++u) {
        const int32_t a = t->unit_ptr[pass][u], b = t->unit_ptr[pass][u + 1];
        append_scope(t->per_unit[pass], merge_runs(slices, t->unit_slices[pass].data() + a, b - a), pass == 1,
                     [&](int32_t sample) -> std::pair<int32_t, int32_t> {
                       int32_t before = 0, after = 0;      // furthest reach of an earlier / a later unit (0: none)
                       for (const auto& ur : reach[sample]) {
                         if (ur.first < u) before = std::max(before, ur.second);
                         if (ur.first > u) after = std::max(after, ur.second);
                       }
                       return {before, after};
                     });
      }
    }
    std::vector<int32_t> all(n_slices);
    for (int32_t i = 0; i < n_slices; ++i) all[i] = i;
    for (int z = 0; z < kNumTileSizes; ++z) { t->fused.q_off[z].push_back(0); t->fused.kv_off[z].push_back(0); }
    for (int ti = 0; ti < kNumSplitTiles; ++ti)
      for (int c = 0; c < kNumSplitClasses; ++c) { t->fused.split_off[ti][c].push_back(0); t->fused.reduce_off[ti][c].push_back(0); }
    append_scope(t->fused, merge_runs(slices, all.data(), n_slices), true,
                 [](int32_t) -> std::pair<int32_t, int32_t> { return {0, 0}; });

    // one blob, one upload
    std::vector<char> blob;
    const size_t off_cu = place(blob, t->cu), off_sl = place(blob, t->slices);
    size_t off_q[3][kNumTileSizes], off_kv[3][kNumTileSizes], off_seg[3], off_sp[3][kNumSplitTiles][kNumSplitClasses], off_rd[3][kNumSplitTiles][kNumSplitClasses];
    ScopeLists* lists[3] = {&t->per_unit[0], &t->per_unit[1], &t->fused};
    for (int s = 0; s < 3; ++s) {
      for (int z = 0; z < kNumTileSizes; ++z) {
        off_q[s][z] = place(blob, lists[s]->q_items[z]);
        off_kv[s][z] = place(blob, lists[s]->kv_items[z]);
      }
      off_seg[s] = place(blob, lists[s]->segs);
      for (int ti = 0; ti < kNumSplitTiles; ++ti)
        for (int c = 0; c < kNumSplitClasses; ++c) {
          off_sp[s][ti][c] = place(blob, lists[s]->split_items[ti][c]);
          off_rd[s][ti][c] = place(blob, lists[s]->reduce_items[ti][c]);
        }
    }
    blob.resize(align_up(blob.size()) + 256);
    hipError_t e = hipGetDevice(&t->device);
    if (e == hipSuccess) (void)prepare_static_scratch();    // set-up for slimattn_bwd_static on this device; its own call reports a failure
    if (e == hipSuccess) e = hipMalloc(&t->d_blob, blob.size());
    if (e == hipSuccess && !use_stream) e = hipMemcpy(t->d_blob, blob.data(), blob.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess && use_stream) {
      // the copy is queued on the caller's stream from a pinned staging buffer that lives as long as the handle:
      // launches queued on the same stream afterwards see the tables, and the host does not wait
      e = hipHostMalloc(&t->h_staging, blob.size(), hipHostMallocDefault);
      if (e == hipSuccess) {
        std::memcpy(t->h_staging, blob.data(), blob.size());
        e = hipMemcpyAsync(t->d_blob, t->h_staging, blob.size(), hipMemcpyHostToDevice, (hipStream_t)stream);
      }
    }
    if (e != hipSuccess) {
      g_last_hip_error = (int)e;
      slimattn_tables_destroy(t);
      return SLIMATTN_EHIP;
    }
    const char* base = (const char*)t->d_blob;
    t->d_cu = (const int32_t*)(base + off_cu);
    t->d_slices = (const slimattn_slice*)(base + off_sl);
    DeviceLists* dl[3] = {&t->d_per_unit[0], &t->d_per_unit[1], &t->d_fused};
    for (int s = 0; s < 3; ++s) {
      for (int z = 0; z < kNumTileSizes; ++z) {
        dl[s]->q_items[z] = (const QItem*)(base + off_q[s][z]);
        dl[s]->kv_items[z] = (const KvItem*)(base + off_kv[s][z]);
      }
      dl[s]->segs = (const Seg*)(base + off_seg[s]);
      for (int ti = 0; ti < kNumSplitTiles; ++ti)
        for (int c = 0; c < kNumSplitClasses; ++c) {
          dl[s]->split_items[ti][c] = (const KvItem*)(base + off_sp[s][ti][c]);
          dl[s]->reduce_items[ti][c] = (const KvReduce*)(base + off_rd[s][ti][c]);
        }
    }
  } catch (const std::bad_alloc&) {
    delete t;
    return SLIMATTN_ENOMEM;
  }
  *out = t;
  return SLIMATTN_OK;
}

void slimattn_tables_destroy(slimattn_tables* t) {
  if (!t) return;
  if (t->d_blob) (void)hipFree(t->d_blob);      // (waits for work that may still read the tables)
  if (t->h_staging) (void)hipHostFree(t->h_staging);
  delete t;
}

int64_t slimattn_tables_count(const slimattn_tables* t, int what) {
  if (!t) return -1;
  switch (what) {
    case 0: return t->total_tokens;
    case 1: return t->n_samples;
    case 2: return t->n_slices;
    case 3: return t->n_units[0];
    case 4: return t->n_units[1];
    case 5: case 6: case 7: case 8: return (int64_t)t->fused.reduce_items[0][what - 5].size();
    default: return -1;
  }
}

int slimattn_bwd_released_rows(const slimattn_tables* t, int32_t unit, int32_t* ranges, int32_t cap, int32_t* n_ranges) {
  if (!t || !n_ranges || cap < 0 || (cap > 0 && !ranges)) return SLIMATTN_EINVAL;
  if (unit < 0 || unit >= t->n_units[1]) return SLIMATTN_EINVAL;
  // per sample: the rows between the furthest reach of a later unit and this unit's own reach
  std::vector<int32_t> mine(t->n_samples, 0), later(t->n_samples, 0);
  for (int32_t u = unit; u < t->n_units[1]; ++u)
    for (int32_t i = t->unit_ptr[1][u]; i < t->unit_ptr[1][u + 1]; ++i) {
      const slimattn_slice& x = t->slices[t->unit_slices[1][i]];
      int32_t& r = (u == unit ? mine : later)[x.sample];
      r = std::max(r, x.q_start + x.q_len);
    }
  std::vector<std::pair<int32_t, int32_t>> merged;
  for (int32_t s = 0; s < t->n_samples; ++s) {
    const int32_t a = std::max(later[s], t->cu[s]), b = mine[s];
    if (b <= a) continue;
    if (!merged.empty() && merged.back().second == a) merged.back().second = b;
    else merged.emplace_back(a, b);
  }
  *n_ranges = (int32_t)merged.size();
  if ((size_t)cap < merged.size()) return SLIMATTN_ECAP;
  for (size_t i = 0; i < merged.size(); ++i) { ranges[2 * i] = merged[i].first; ranges[2 * i + 1] = merged[i].second; }
  return SLIMATTN_OK;
}

size_t slimattn_bwd_workspace_bytes(const slimattn_tables* t, int32_t hq, int32_t hkv, int32_t d) {
  if (!t || hq < 1 || hkv < 1 || d < 1) return 0;
  const size_t T = (size_t)t->total_tokens;
  const int c = split_class(hkv);
  size_t parts = 0;                       // the larger of the two tile sizes' needs (which kernel runs depends on dtype, d)
  for (int ti = 0; ti < kNumSplitTiles; ++ti) {
    const size_t slots = (size_t)std::max({t->per_unit[0].max_slots[ti][c], t->per_unit[1].max_slots[ti][c], t->fused.max_slots[ti][c]});
    parts = std::max(parts, slots * hkv * 2 * kSplitTileRows[ti] * d * sizeof(float));
  }
  return align_up(2 * T * hkv * d * sizeof(float)) + align_up(T * hq * sizeof(float)) + align_up(T * hq * 16) + align_up(parts) + 256;
}

}  // extern "C"
