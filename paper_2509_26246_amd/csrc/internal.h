// Private declarations shared by the host builder, the table handle and the kernel launchers.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/slimattn.h"

namespace slimattn {

// Tile sizes for which work-lists are derived: query tiles of 64 (fp32 kernels) and 128 rows (bf16 forward,
// dQ), key tiles of 64 (fp32) and 256 rows (bf16 dK/dV).
constexpr int kNumTileSizes = 3;
constexpr int kTileSizes[kNumTileSizes] = {64, 128, 256};
inline bool is_query_tile(int rows) { return rows == 64 || rows == 128; }
inline bool is_key_tile(int rows) { return rows == 64 || rows == 256; }
inline int tile_index(int rows) {
  for (int i = 0; i < kNumTileSizes; ++i) if (kTileSizes[i] == rows) return i;
  return -1;
}

// A query tile: rows [q_row0, q_row0 + q_rows) of one sample whose first token is kv_start.
// Row i sees keys kv_start .. i.  The tile therefore needs keys [kv_start, q_row0 + q_rows).
struct QItem { int32_t q_row0, q_rows, kv_start, pad; };

// A run of query rows [q_lo, q_hi) of one sample that belong to the launch scope.
struct Seg { int32_t q_lo, q_hi; };

// A key tile: rows [kv_row0, kv_row0 + kv_rows) of one sample, and the scope's query runs of that
// sample that end after kv_row0 (segs[seg_begin .. seg_end), ascending).  slot < 0: the item covers
// every such run and its block owns the tile's dK/dV.  slot >= 0: the item is one part of a heavy
// tile whose query rows were divided among several blocks; it covers only its own runs and stores
// its sums as fp32 partial tile number `slot`, which a reduction launch adds up in slot order.
// load_until, final_from: where the rows' sums come from and go to (below).
struct KvItem { int32_t kv_row0, kv_rows, seg_begin, seg_end, slot, load_until, final_from, pad; };

// A key row collects from every unit of the backward list that has query rows of the sample at or after it
// (a slice's dK/dV are complete only when all later slices have run: the paper's inter-slice dependency of
// the backward pass).  Units run in list order, and a unit reaches the rows before the end of its last query
// row in the sample.  So for the rows of a unit's key tile: rows below `load_until` (the furthest reach of an
// earlier unit) continue a partial sum that unit left in the fp32 accumulators, the others start from zero
// (nothing has to be cleared beforehand); rows from `final_from` on (the furthest reach of a later unit) get no
// further contribution and are written as dK/dV in the output type, the others go to the accumulators.  A
// row's gradient is thus released by its last contributor, not at the end of the list.  Whole-list scope:
// load_until = 0, final_from = 0.

// A divided key tile: partial tiles first_slot .. first_slot + n_parts - 1 are its parts.
struct KvReduce { int32_t kv_row0, kv_rows, first_slot, n_parts, load_until, final_from, pad0, pad1; };

// Divided lists exist for the 256-row key tile (the bf16 dK/dV kernel) and four classes
// of KV-head count (1, 2, 4, >= 8): a launch has items x KV heads blocks, so the fewer KV heads, the
// fewer blocks share the work and the more a single long sample's first tiles dominate the makespan.
constexpr int kNumSplitTiles = 1;                               // key-tile sizes for which divided lists are built
constexpr int kSplitTileRows[kNumSplitTiles] = {256};           // the bf16 dK/dV kernel's tile
// Slots the per-slot share of the work is taken over: 3/4 of the kernel's 256 resident blocks (measured: a
// part costs a V tile, K fragments and an fp32 partial tile to set up, and dividing more finely lost 1-4 %).
constexpr int kSplitBlockSlots[kNumSplitTiles] = {192};
inline int split_tile_index(int rows) { return rows == 256 ? 0 : -1; }
constexpr int kNumSplitClasses = 4;
inline int split_class(int n_kv_heads) { return n_kv_heads >= 8 ? 3 : n_kv_heads >= 4 ? 2 : n_kv_heads >= 2 ? 1 : 0; }

// A launch scope is either one unit or the whole list ("fused").  Its items are stored heavy-first.
struct ScopeLists {
  std::vector<int32_t> q_off[kNumTileSizes];    // per-unit offsets into q_items (size n_units + 1)
  std::vector<QItem> q_items[kNumTileSizes];    // unit-major, each unit heavy-first
  std::vector<int32_t> kv_off[kNumTileSizes];
  std::vector<KvItem> kv_items[kNumTileSizes];
  std::vector<Seg> segs;                        // all units' runs (and the parts' cut runs), referenced by the items
  // key tiles with heavy tiles divided, per tile size and KV-head class; same unit-major layout
  std::vector<int32_t> split_off[kNumSplitTiles][kNumSplitClasses];
  std::vector<KvItem> split_items[kNumSplitTiles][kNumSplitClasses];
  std::vector<int32_t> reduce_off[kNumSplitTiles][kNumSplitClasses];
  std::vector<KvReduce> reduce_items[kNumSplitTiles][kNumSplitClasses];
  int32_t max_slots[kNumSplitTiles][kNumSplitClasses] = {{0, 0, 0, 0}};   // most partial tiles any one scope needs
};

struct DeviceLists {                            // device mirrors (pointers into one allocation)
  const QItem* q_items[kNumTileSizes];
  const KvItem* kv_items[kNumTileSizes];
  const Seg* segs;
  const KvItem* split_items[kNumSplitTiles][kNumSplitClasses];
  const KvReduce* reduce_items[kNumSplitTiles][kNumSplitClasses];
};

}  // namespace slimattn

struct slimattn_tables {
  int32_t n_samples = 0, n_slices = 0, n_units[2] = {0, 0};
  int64_t total_tokens = 0;
  int32_t max_sample_len = 0;
  std::vector<int32_t> cu;
  std::vector<slimattn_slice> slices;
  std::vector<int32_t> unit_ptr[2], unit_slices[2];      // [0] forward list, [1] backward list
  slimattn::ScopeLists per_unit[2];                       // one scope per unit of each list
  slimattn::ScopeLists fused;                             // one scope: every slice (same for both passes)
  slimattn::DeviceLists d_per_unit[2], d_fused;
  const int32_t* d_cu = nullptr;
  const slimattn_slice* d_slices = nullptr;
  void* d_blob = nullptr;
  void* h_staging = nullptr;      // pinned copy of the tables for an upload queued on a stream (kept until destroy)
  int device = -1;
};

namespace slimattn {

struct LaunchCtx {
  const slimattn_params* p;
  void* stream;           // hipStream_t
  int64_t T;
};

// Kernel launchers (defined in the .hip files).  Each returns a hipError_t as int.
int launch_fwd_f32(const LaunchCtx&, const float* q, const float* k, const float* v, float* o, float* lse,
                   const QItem* items, int n_items);
// delta = rowsum(dO * O) for the rows of the listed query tiles
int launch_bwd_delta_f32(const LaunchCtx&, const float* o, const float* dO, float* delta, const QItem* items, int n_items);
int launch_bwd_dq_f32(const LaunchCtx&, const float* q, const float* k, const float* v, const float* dO, const float* lse,
                      const float* delta, float* dQ, const QItem* items, int n_items);
int launch_bwd_dkdv_f32(const LaunchCtx&, const float* q, const float* k, const float* v, const float* dO, const float* lse,
                        const float* delta, float* acc_dk, float* acc_dv, float* dK, float* dV, const KvItem* items,
                        int n_items, const Seg* segs);

int launch_fwd_bf16(const LaunchCtx&, const void* q, const void* k, const void* v, void* o, float* lse,
                    const QItem* items, int n_items);
// even group sizes at head dim 128: one wave per SIMD, two heads per wave (fwd_wide_bf16.hip); same arguments
int launch_fwd_wide_bf16(const LaunchCtx&, const void* q, const void* k, const void* v, void* o, float* lse,
                         const QItem* items, int n_items);
// Row statistics of the bf16 backward (-lse*log2e and -delta = -dO.O per row and head, as bf16 triples):
// either the dQ kernel computes and stores them for the rows it owns (own_stats != 0; `o`, `lse` read), or
// the prepass below has stored them for the rows of the same query tiles and the dQ kernel reads them
// (own_stats == 0).  Either way only rows of the launch scope are read.
int launch_bwd_stat_bf16(const LaunchCtx&, const void* o, const void* dO, const float* lse, void* stat3, const QItem* items,
                         int n_items);
int launch_bwd_dq_bf16(const LaunchCtx&, const void* q, const void* k, const void* v, const void* dO, const void* o,
                       const float* lse, void* stat3, int own_stats, void* dQ, const QItem* items, int n_items);
// head_dim 128: one wave per SIMD, 256 key rows per block (dkdv_wide_bf16.hip); same arguments
int launch_bwd_dkdv_wide_bf16(const LaunchCtx&, const void* q, const void* k, const void* v, const void* dO, const void* stat3,
                            float* acc_dk, float* acc_dv, void* dK, void* dV, const KvItem* items, int n_items, const Seg* segs,
                            float* parts);
// adds up the partial tiles (tile_rows rows each) of divided key tiles, in slot order, into dK/dV or the
// fp32 accumulators
int launch_bwd_reduce_bf16(const LaunchCtx&, const float* parts, float* acc_dk, float* acc_dv, void* dK, void* dV,
                           const KvReduce* items, int n_items, int tile_rows);

// Looks up the built-in scratch array of slimattn_bwd_static on the current device (so that the first such call
// finds it ready); returns a SLIMATTN_* code.
int prepare_static_scratch();

// Tile sizes each kernel family uses (must be one of kTileSizes).
int fwd_q_tile(int dtype, int head_dim);
int dq_q_tile(int dtype, int head_dim);
int dkdv_kv_tile(int dtype, int head_dim);
}  // namespace slimattn
