// Entry points slimattn_fwd / slimattn_bwd: argument checks, scope selection, launches.
// No device allocation and no synchronisation happens here.
#include <hip/hip_runtime.h>

#include <mutex>
#include <vector>

#include "internal.h"

// Built-in scratch for slimattn_bwd_static: one array per GPU the library runs on, held until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels and fills get the
// device address looked up once per device (each device has its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[SLIMATTN_STATIC_SCRATCH_BYTES];

namespace slimattn {
int& last_hip_error();

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up at the first call on that device).
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { last_hip_error() = (int)e; return SLIMATTN_EHIP; }
  if (dev < 0 || dev >= kMaxDevices) return SLIMATTN_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { last_hip_error() = (int)e; return SLIMATTN_EHIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SLIMATTN_OK;
}

bool aligned16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_common(const slimattn_params* p, const slimattn_tables* t, int pass, int* lo, int* hi) {
  if (!p || !t) return SLIMATTN_EINVAL;
  if ((int64_t)p->total_tokens != t->total_tokens) return SLIMATTN_EINVAL;
  const int rc = slimattn_shape_supported(p->total_tokens, t->max_sample_len, p->n_q_heads, p->n_kv_heads, p->head_dim, p->dtype);
  if (rc != SLIMATTN_OK) return rc;
  if (!(p->scale == p->scale)) return SLIMATTN_EINVAL;
  *lo = p->unit_lo;
  *hi = p->unit_hi < 0 ? t->n_units[pass] : p->unit_hi;
  if (*lo < 0 || *hi > t->n_units[pass] || *lo > *hi) return SLIMATTN_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != t->device) return SLIMATTN_EINVAL;
  return SLIMATTN_OK;
}

int hip_rc(int e) {
  if (e == 0) return SLIMATTN_OK;
  last_hip_error() = e;
  return SLIMATTN_EHIP;
}

size_t align_up(size_t x) { return (x + 255) & ~size_t(255); }

// Optional per-launch timing (slimattn_profile_enable).  Events are created up front; recording
// an event allocates nothing.  A launch that finds the pool used up runs untimed and is counted as dropped.
struct Profiler {
  std::vector<hipEvent_t> start, stop;
  std::vector<int> cls, pass, unit;
  size_t used = 0;
  int64_t dropped = 0;
  bool on = false;
  int cur_pass = 0, cur_unit = -1;      // what the launches being issued belong to (set by the entry points)
} g_prof;

template <class F>
int timed(int cls, void* stream, F&& launch) {
  if (!g_prof.on) return launch();
  if (g_prof.used >= g_prof.start.size()) { ++g_prof.dropped; return launch(); }
  const size_t i = g_prof.used++;
  g_prof.cls[i] = cls;
  g_prof.pass[i] = g_prof.cur_pass;
  g_prof.unit[i] = g_prof.cur_unit;
  (void)hipEventRecord(g_prof.start[i], (hipStream_t)stream);
  const int e = launch();
  (void)hipEventRecord(g_prof.stop[i], (hipStream_t)stream);
  return e;
}

// The whole call between two events on the caller's stream (the gaps between its launches included, so this is
// the time a caller sees, not the sum of the kernels' times).
template <class F>
int timed_call(int cls, void* stream, F&& body) {
  if (!g_prof.on) return body();
  if (g_prof.used >= g_prof.start.size()) { ++g_prof.dropped; return body(); }
  const size_t i = g_prof.used++;
  g_prof.cls[i] = cls;
  g_prof.pass[i] = g_prof.cur_pass;
  g_prof.unit[i] = -1;
  (void)hipEventRecord(g_prof.start[i], (hipStream_t)stream);
  const int rc = body();
  (void)hipEventRecord(g_prof.stop[i], (hipStream_t)stream);
  return rc;
}

}  // namespace

int prepare_static_scratch() {
  void* p = nullptr;
  return static_scratch(&p);
}

}  // namespace slimattn

using namespace slimattn;

extern "C" {

int slimattn_shape_supported(int64_t total_tokens, int32_t max_sample_len, int32_t n_q_heads, int32_t n_kv_heads,
                             int32_t head_dim, int32_t dtype) {
  if (dtype != SLIMATTN_F32 && dtype != SLIMATTN_BF16) return SLIMATTN_EINVAL;
  if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 || n_q_heads > 65535) return SLIMATTN_EINVAL;
  const int d = head_dim;
  if (dtype == SLIMATTN_BF16 ? !(d == 64 || d == 128) : !(d == 16 || d == 32 || d == 64 || d == 128)) return SLIMATTN_EINVAL;
  if (total_tokens < 0 || total_tokens > INT32_MAX || max_sample_len < 0 || max_sample_len > total_tokens) return SLIMATTN_EINVAL;
  if (dtype == SLIMATTN_BF16) {
    // The bf16 kernels address tile rows with 32-bit byte offsets from a base that moves with the work item: the
    // sample's first row (K, V, with Hkv heads per row) or the key tile's first row (Q, dO, with Hq heads per
    // row).  The largest offset is therefore one sample's rows times the wider row, and it has to stay below
    // 2^31 (the offsets are formed in signed 32-bit arithmetic).  The pack as a whole may be larger: pointers
    // to a work item's base are 64-bit.
    if ((int64_t)max_sample_len * n_q_heads * d * 2 >= (int64_t(1) << 31)) return SLIMATTN_EINVAL;
    // row statistics of the backward pass: 16 bytes per (head, token), one 32-bit offset from the array's start
    if (total_tokens * n_q_heads * 16 >= (int64_t(1) << 31)) return SLIMATTN_EINVAL;
  }
  return SLIMATTN_OK;
}

static int fwd_impl(const slimattn_params* p, const void* q, const void* k, const void* v, const slimattn_tables* t, void* o,
                    float* lse, void* stream, int lo, int hi);

int slimattn_fwd(const slimattn_params* p, const void* q, const void* k, const void* v, const slimattn_tables* t,
                 void* o, float* lse, void* stream) {
  int lo, hi;
  int rc = check_common(p, t, 0, &lo, &hi);
  if (rc != SLIMATTN_OK) return rc;
  if (t->total_tokens == 0 || lo == hi) return SLIMATTN_OK;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse)) return SLIMATTN_EINVAL;
  g_prof.cur_pass = 0;
  g_prof.cur_unit = -1;
  return timed_call(SLIMATTN_K_FWD_CALL, stream, [&] { return fwd_impl(p, q, k, v, t, o, lse, stream, lo, hi); });
}

static int fwd_impl(const slimattn_params* p, const void* q, const void* k, const void* v, const slimattn_tables* t, void* o,
                    float* lse, void* stream, int lo, int hi) {
  int rc = SLIMATTN_OK;
  const int z = tile_index(fwd_q_tile(p->dtype, p->head_dim));
  const LaunchCtx ctx{p, stream, t->total_tokens};
  auto run = [&](const QItem* items, int n) -> int {
    return timed(SLIMATTN_K_FWD, stream, [&] {
      return p->dtype == SLIMATTN_F32
                 ? launch_fwd_f32(ctx, (const float*)q, (const float*)k, (const float*)v, (float*)o, lse, items, n)
                 : launch_fwd_bf16(ctx, q, k, v, o, lse, items, n);
    });
  };
  const bool whole = lo == 0 && hi == t->n_units[0];
  g_prof.cur_pass = 0;
  g_prof.cur_unit = -1;
  if (whole && !(p->flags & SLIMATTN_FLAG_PER_UNIT_LAUNCH))
    return hip_rc(run(t->d_fused.q_items[z], (int)t->fused.q_items[z].size()));
  const auto& off = t->per_unit[0].q_off[z];
  if (!(p->flags & SLIMATTN_FLAG_PER_UNIT_LAUNCH))
    return hip_rc(run(t->d_per_unit[0].q_items[z] + off[lo], off[hi] - off[lo]));
  for (int u = lo; u < hi; ++u) {
    g_prof.cur_unit = u;
    rc = hip_rc(run(t->d_per_unit[0].q_items[z] + off[u], off[u + 1] - off[u]));
    if (rc != SLIMATTN_OK) return rc;
  }
  return SLIMATTN_OK;
}

static int bwd_impl(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o, const float* lse,
                    const void* dO, const slimattn_tables* t, void* dQ, void* dK, void* dV, void* workspace, void* stream, int lo,
                    int hi);

int slimattn_bwd(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o, const float* lse,
                 const void* dO, const slimattn_tables* t, void* dQ, void* dK, void* dV, void* workspace, void* stream) {
  int lo, hi;
  int rc = check_common(p, t, 1, &lo, &hi);
  if (rc != SLIMATTN_OK) return rc;
  if (t->total_tokens == 0 || lo == hi) return SLIMATTN_OK;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(dO) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return SLIMATTN_EINVAL;
  g_prof.cur_pass = 1;
  g_prof.cur_unit = -1;
  return timed_call(SLIMATTN_K_BWD_CALL, stream,
                    [&] { return bwd_impl(p, q, k, v, o, lse, dO, t, dQ, dK, dV, workspace, stream, lo, hi); });
}

static int bwd_impl(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o, const float* lse,
                    const void* dO, const slimattn_tables* t, void* dQ, void* dK, void* dV, void* workspace, void* stream, int lo,
                    int hi) {
  int rc = SLIMATTN_OK;
  const bool f32 = p->dtype == SLIMATTN_F32;
  const size_t T = (size_t)t->total_tokens;
  const size_t acc_elems = T * p->n_kv_heads * p->head_dim;
  float* acc_dk = (float*)workspace;
  float* acc_dv = acc_dk + acc_elems;
  float* delta = (float*)((char*)workspace + align_up(2 * acc_elems * sizeof(float)));
  // bf16 path: -lse*log2e and -delta as bf16 triples, 16 bytes per row and head (written by the dQ kernel, read by the dK/dV kernel)
  void* stat3 = (char*)delta + align_up(T * p->n_q_heads * sizeof(float));
  float* parts = (float*)((char*)stat3 + align_up(T * p->n_q_heads * 16));              // partial tiles of divided key tiles
  const int sc = split_class(p->n_kv_heads);
  const int n_units = t->n_units[1];
  const bool whole = lo == 0 && hi == n_units;
  const bool per_unit = (p->flags & SLIMATTN_FLAG_PER_UNIT_LAUNCH) != 0;

  const LaunchCtx ctx{p, stream, t->total_tokens};

  // Row statistic delta_i = dO_i . o_i, always for the query rows of the launch scope only (a caller that runs the
  // list one unit at a time need not have o, lse and dO of later units yet).  fp32: a prepass in front of each dQ
  // launch.  bf16: normally the dQ kernel computes it for the rows it owns and stores it (with lse in log2 units,
  // both as bf16 triples) for the dK/dV launch of the same scope, which therefore runs after it; with a very
  // long sample (its K and V, over all KV heads, far beyond what the caches hold) the dQ blocks depend on
  // streaming the same K/V tiles at the same time, and the longer prologue cost 9 % there (256K sample), so
  // the prepass is kept.  (The dQ launch on a second stream beside the dK/dV launch, with the statistics always
  // from the prepass, was measured: the two kernels cannot share a compute unit and only slow each other --
  // 32K pack, fused 928 -> 893 TFLOP/s, per-unit 734 -> 716 -- so every launch stays on the caller's stream.)
  const bool own_stats = !f32 && !(p->flags & SLIMATTN_FLAG_STATS_PREPASS) &&
                         (size_t)t->max_sample_len * p->n_kv_heads * p->head_dim * 4 <= (size_t(128) << 20);
  const int zq = tile_index(dq_q_tile(p->dtype, p->head_dim));
  const int zk = tile_index(dkdv_kv_tile(p->dtype, p->head_dim));
  auto run_dq = [&](const QItem* items, int n) -> int {
    if (!own_stats) {
      const int e = timed(SLIMATTN_K_DELTA, stream, [&] {
        return f32 ? launch_bwd_delta_f32(ctx, (const float*)o, (const float*)dO, delta, items, n)
                   : launch_bwd_stat_bf16(ctx, o, dO, lse, stat3, items, n);
      });
      if (e != 0) return e;
    }
    return timed(SLIMATTN_K_DQ, stream, [&] {
      return f32 ? launch_bwd_dq_f32(ctx, (const float*)q, (const float*)k, (const float*)v, (const float*)dO, lse, delta,
                                     (float*)dQ, items, n)
                 : launch_bwd_dq_bf16(ctx, q, k, v, dO, o, lse, stat3, own_stats ? 1 : 0, dQ, items, n);
    });
  };
  auto run_dkdv = [&](const KvItem* items, int n, const Seg* segs) -> int {
    return timed(SLIMATTN_K_DKDV, stream, [&] {
      return f32 ? launch_bwd_dkdv_f32(ctx, (const float*)q, (const float*)k, (const float*)v, (const float*)dO, lse,
                                       delta, acc_dk, acc_dv, (float*)dK, (float*)dV, items, n, segs)
                 : launch_bwd_dkdv_wide_bf16(ctx, q, k, v, dO, stat3, acc_dk, acc_dv, dK, dV, items, n, segs, parts);
    });
  };
  // bf16: the key-tile list in which heavy tiles are divided among several blocks, followed by the
  // launch that adds the parts up (a scope without divided tiles has an empty reduction list)
  auto run_dkdv_split = [&](const ScopeLists& L, const DeviceLists& D, int u) -> int {
    const int tile_rows = dkdv_kv_tile(p->dtype, p->head_dim), ti = split_tile_index(tile_rows);
    const int a = L.split_off[ti][sc][u], b = L.split_off[ti][sc][u + 1];
    int e = run_dkdv(D.split_items[ti][sc] + a, b - a, D.segs);
    if (e != 0) return e;
    const int ra = L.reduce_off[ti][sc][u], rb = L.reduce_off[ti][sc][u + 1];
    if (rb == ra) return 0;
    return timed(SLIMATTN_K_REDUCE, stream, [&] {
      return launch_bwd_reduce_bf16(ctx, parts, acc_dk, acc_dv, dK, dV, D.reduce_items[ti][sc] + ra, rb - ra, tile_rows);
    });
  };
  auto finish = [&](int e) -> int { return hip_rc(e); };

  if (whole && !per_unit) {
    // One scope holding every slice: each key tile's owner sums all later query rows itself and
    // writes dK/dV directly; the fp32 accumulators in the workspace are not touched.
    int e = run_dq(t->d_fused.q_items[zq], (int)t->fused.q_items[zq].size());
    if (e == 0)
      e = f32 ? run_dkdv(t->d_fused.kv_items[zk], (int)t->fused.kv_items[zk].size(), t->d_fused.segs)
              : run_dkdv_split(t->fused, t->d_fused, 0);
    return finish(e);
  }

  const auto& qoff = t->per_unit[1].q_off[zq];
  const auto& koff = t->per_unit[1].kv_off[zk];
  int e = 0;
  if (!per_unit) e = run_dq(t->d_per_unit[1].q_items[zq] + qoff[lo], qoff[hi] - qoff[lo]);
  for (int u = lo; u < hi && e == 0; ++u) {
    // Units run one after another on the stream; each adds its queries' contributions to every key row of the
    // prefix it sees.  A row's single owner block continues from the fp32 accumulator an earlier unit left
    // (the row's first unit starts from zero, so nothing has to be cleared) and the row's last unit writes
    // dK/dV themselves: the summation order is the unit order, and a row is released as soon as it is complete.
    g_prof.cur_unit = u;
    if (per_unit) e = run_dq(t->d_per_unit[1].q_items[zq] + qoff[u], qoff[u + 1] - qoff[u]);
    if (e == 0)
      e = f32 ? run_dkdv(t->d_per_unit[1].kv_items[zk] + koff[u], koff[u + 1] - koff[u], t->d_per_unit[1].segs)
              : run_dkdv_split(t->per_unit[1], t->d_per_unit[1], u);
  }
  g_prof.cur_unit = -1;
  rc = finish(e);
  return rc;
}

int slimattn_bwd_static(const slimattn_params* p, const void* q, const void* k, const void* v, const void* o, const float* lse,
                        const void* dO, const slimattn_tables* t, void* dQ, void* dK, void* dV, void* stream) {
  if (!p || !t) return SLIMATTN_EINVAL;
  if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->head_dim < 1) return SLIMATTN_EINVAL;
  const size_t need = slimattn_bwd_workspace_bytes(t, p->n_q_heads, p->n_kv_heads, p->head_dim);
  if (need == 0 || need > (size_t)SLIMATTN_STATIC_SCRATCH_BYTES) return SLIMATTN_ESCRATCH;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != SLIMATTN_OK) return rc;
  return slimattn_bwd(p, q, k, v, o, lse, dO, t, dQ, dK, dV, ws, stream);
}

int slimattn_profile_enable(int32_t max_launches) {
  for (hipEvent_t e : g_prof.start) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_prof.stop) (void)hipEventDestroy(e);
  g_prof.start.clear();
  g_prof.stop.clear();
  g_prof.cls.clear();
  g_prof.pass.clear();
  g_prof.unit.clear();
  g_prof.used = 0;
  g_prof.dropped = 0;
  g_prof.on = false;
  if (max_launches <= 0) return SLIMATTN_OK;
  g_prof.start.resize(max_launches);
  g_prof.stop.resize(max_launches);
  g_prof.cls.assign(max_launches, 0);
  g_prof.pass.assign(max_launches, 0);
  g_prof.unit.assign(max_launches, -1);
  for (int32_t i = 0; i < max_launches; ++i) {
    hipError_t e = hipEventCreate(&g_prof.start[i]);
    if (e == hipSuccess) e = hipEventCreate(&g_prof.stop[i]);
    if (e != hipSuccess) return hip_rc((int)e);
  }
  g_prof.on = true;
  return SLIMATTN_OK;
}

int slimattn_profile_read_launches(int32_t cap, int32_t* cls, int32_t* pass, int32_t* unit, float* ms, int32_t* n_launches,
                                   int64_t* dropped) {
  if (!n_launches || cap < 0 || (cap > 0 && (!cls || !pass || !unit || !ms))) return SLIMATTN_EINVAL;
  *n_launches = (int32_t)g_prof.used;
  if (dropped) *dropped = g_prof.dropped;
  if ((size_t)cap < g_prof.used) return SLIMATTN_ECAP;
  for (size_t i = 0; i < g_prof.used; ++i) {
    hipError_t e = hipEventSynchronize(g_prof.stop[i]);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, g_prof.start[i], g_prof.stop[i]);
    if (e != hipSuccess) return hip_rc((int)e);
    cls[i] = g_prof.cls[i];
    pass[i] = g_prof.pass[i];
    unit[i] = g_prof.unit[i];
    ms[i] = t;
  }
  g_prof.used = 0;
  g_prof.dropped = 0;
  return SLIMATTN_OK;
}

int slimattn_profile_read(double* ms, int64_t* launches) {
  if (!ms || !launches) return SLIMATTN_EINVAL;
  for (int c = 0; c < SLIMATTN_K_COUNT; ++c) { ms[c] = 0.0; launches[c] = 0; }
  for (size_t i = 0; i < g_prof.used; ++i) {
    hipError_t e = hipEventSynchronize(g_prof.stop[i]);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, g_prof.start[i], g_prof.stop[i]);
    if (e != hipSuccess) return hip_rc((int)e);
    ms[g_prof.cls[i]] += t;
    launches[g_prof.cls[i]]++;
  }
  const bool lost = g_prof.dropped > 0;
  g_prof.used = 0;
  g_prof.dropped = 0;
  return lost ? SLIMATTN_ECAP : SLIMATTN_OK;
}

}  // extern "C"
