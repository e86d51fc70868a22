// Device helpers for the bf16 MFMA kernels (gfx950): vector types, swizzled LDS tiles, fragment
// reads in both orientations, global<->LDS staging.
//
// MFMA 32x32x16 bf16 operand layout (lane l, half = l / 32, n = l % 32):
//   A[m = n][k = 8*half + t], B[k = 8*half + t][n], t = 0..7 (eight consecutive k per lane);
//   C[i = 8*(r/4) + 4*half + (r%4)][j = n], r = 0..15.
// A product's C registers r = 8e .. 8e+7 therefore hold, for a fixed column, the rows
// {16e + 4*half + 0..3} and {16e + 8 + 4*half + 0..3}; used as the next product's B operand they
// fix which row each k-slot stands for, and the A operand of that product is read to match
// (transposed LDS reads below).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slimattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __bf16 bf16;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

// Swizzled LDS tile of ROWS x D bf16 (no padding).  The 16-byte unit index is XORed with a
// function of the row so that (a) 16 consecutive rows at one column and (b) 4 consecutive rows
// x 4 consecutive units both touch 16 distinct units of a 256-byte bank line.
template <int D>
__device__ __forceinline__ int lds_off16(int row, int unit);
template <>
__device__ __forceinline__ int lds_off16<128>(int row, int unit) {
  const int f = ((row & 3) << 2) | ((row >> 2) & 3);
  return row * 256 + ((unit ^ f) << 4);
}
template <>
__device__ __forceinline__ int lds_off16<64>(int row, int unit) {
  const int R = row >> 1;
  const int f = ((R & 1) << 2) | ((R >> 1) & 3);
  const int u = ((row & 1) << 3) | unit;
  return R * 256 + ((u ^ f) << 4);
}

// Pack eight fp32 accumulators (registers r0 .. r0+7 of a C tile) into a bf16 B operand
// (four packed round-to-nearest-even conversions).
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float floatx8;
__device__ __forceinline__ bf16x8 pack8(const floatx16& c, int r0) {
  floatx8 t;
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] = c[r0 + i];
  return __builtin_convertvector(t, bf16x8);
}

// Fragment of eight bf16 values times a scalar, rounded back to bf16 (used to fold the softmax
// scale, in log2 units, into one operand of the score product).
__device__ __forceinline__ bf16x8 scale8(bf16x8 a, float c) {
  floatx8 t = __builtin_convertvector(a, floatx8);
#pragma unroll
  for (int i = 0; i < 8; ++i) t[i] *= c;
  return __builtin_convertvector(t, bf16x8);
}

// Sum of the eight bf16 values of a fragment, added to acc (four dot-products against ones).
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
__device__ __forceinline__ float sum8(bf16x8 a, float acc) {
  const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    bf16x2 pr = {a[2 * i], a[2 * i + 1]};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
  }
  return acc;
}

// Software-pipelined operand stream: N fragments, each read from LDS kPre steps before the
// product that consumes it.  `load(i)` returns fragment i, `use(i, frag)` issues its products.
// The trailing scheduling directives pin the order "kPre reads, then (products, read) ...";
// rpf = LDS read instructions per fragment, upf = products per fragment.
template <int N, int kPre, int rpf, int upf, class Load, class Use>
__device__ __forceinline__ void frag_pipeline(Load&& load, Use&& use) {
  decltype(load(0)) fr[N];
#pragma unroll
  for (int i = 0; i < N + kPre; ++i) {
    if (i < N) fr[i] = load(i);
    if (i >= kPre) use(i - kPre, fr[i - kPre]);
  }
  __builtin_amdgcn_sched_group_barrier(0x100, rpf * kPre, 0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, upf, 0);
    if (i + kPre < N) __builtin_amdgcn_sched_group_barrier(0x100, rpf, 0);
  }
}

// ---- LDS fragment pointers kept in registers --------------------------------------------------
// The swizzle makes a fragment's LDS address a non-additive function of (lane, column block), so
// the per-lane addresses are computed once, kept in registers (laundered through an empty asm so
// the compiler does not recompute them at every use) and advanced by adding uniform byte offsets:
// rows are additive, and so is the buffer switch.
typedef LDS_PTR(const char) lds_cptr;

__device__ __forceinline__ lds_cptr keep(lds_cptr p) {
  asm volatile("" : "+v"(p));
  return p;
}
template <int D>
__device__ __forceinline__ lds_cptr lds_row_ptr(lds_cptr tile, int row, int col0) {
  return keep(tile + lds_off16<D>(row, col0 >> 3));
}
// Transposed fragment for an A operand with m = column, k = row: lane l receives, for column
// col0 + (l % 32), the rows {row0 + 4*half + 0..3} and {row0 + 8 + 4*half + 0..3}.  It is built
// from two LDS transpose loads; in each, the 16 lanes of a group supply the addresses of 4 rows x
// 4 chunks of 4 columns, and lane i gets column i of the four rows.  These are the two addresses
// for row0 = 0: p0 serves rows {4*half + 0..3}, p1 rows {8 + 4*half + 0..3}; a fragment at
// row0 = 16*s is read at both pointers + 16*s*(2*D) bytes.
template <int D>
__device__ __forceinline__ void lds_tr_ptrs(lds_cptr tile, int col0, int lane, lds_cptr& p0, lds_cptr& p1) {
  const int i = lane & 15, grp = lane >> 4;
  const int row = 4 * (grp >> 1) + (i >> 2);
  const int col = col0 + 16 * (grp & 1) + 4 * (i & 3);
  p0 = keep(tile + lds_off16<D>(row, col >> 3) + ((col & 4) << 1));
  p1 = keep(tile + lds_off16<D>(row + 8, col >> 3) + ((col & 4) << 1));
}
__device__ __forceinline__ bf16x8 lds_ld_row(lds_cptr p, int byte_off) {
  return *reinterpret_cast<LDS_PTR(const bf16x8)>(p + byte_off);
}
// ---- transposed fragment stream through inline asm ---------------------------------------------
// The compiler's wait-count insertion treats an LDS transpose load as possibly reading what an
// outstanding direct global->LDS load is still writing and puts a full vmcnt(0) wait in front of
// it, which would serialise each tile behind the prefetch of the next one.  The prefetch targets
// the other buffer, so the transpose loads are issued from inline asm, in batches of four
// fragments (eight loads), with the wait counts written by hand: a batch is issued, then
// lgkmcnt(8) waits for everything older than it -- LDS operations complete in order -- which
// makes the previous batch ready while this one is still in flight.  The previous batch is
// passed through the asm as an in/out operand so that its consumers are ordered after the wait.
struct Tr4 { short4v r[8]; };     // four fragments; fragment j = (r[2j], r[2j+1])

__device__ __forceinline__ bf16x8 tr4_frag(const Tr4& t, int j) {
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8v;
  short8v x = __builtin_shufflevector(t.r[2 * j], t.r[2 * j + 1], 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, x);
}
#define SLIMATTN_TR4_READS                                   \
  "ds_read_b64_tr_b16 %0, %[p0] offset:%[o0]\n\t"            \
  "ds_read_b64_tr_b16 %1, %[p1] offset:%[o0]\n\t"            \
  "ds_read_b64_tr_b16 %2, %[p0] offset:%[o1]\n\t"            \
  "ds_read_b64_tr_b16 %3, %[p1] offset:%[o1]\n\t"            \
  "ds_read_b64_tr_b16 %4, %[p0] offset:%[o2]\n\t"            \
  "ds_read_b64_tr_b16 %5, %[p1] offset:%[o2]\n\t"            \
  "ds_read_b64_tr_b16 %6, %[p0] offset:%[o3]\n\t"            \
  "ds_read_b64_tr_b16 %7, %[p1] offset:%[o3]\n\t"
// Issue the four fragments at byte offsets O0..O3 from the fragment address pair (p0, p1).
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void tr4_issue(lds_cptr p0, lds_cptr p1, Tr4& n) {
  asm volatile(SLIMATTN_TR4_READS
               : "=&v"(n.r[0]), "=&v"(n.r[1]), "=&v"(n.r[2]), "=&v"(n.r[3]), "=&v"(n.r[4]), "=&v"(n.r[5]), "=&v"(n.r[6]),
                 "=&v"(n.r[7])
               : [p0] "v"(p0), [p1] "v"(p1), [o0] "n"(O0), [o1] "n"(O1), [o2] "n"(O2), [o3] "n"(O3));
}
// Issue the next batch, then wait until the previous batch `p` has landed.
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void tr4_issue_wait(lds_cptr p0, lds_cptr p1, Tr4& n, Tr4& p) {
  asm volatile(SLIMATTN_TR4_READS "s_waitcnt lgkmcnt(8)"
               : "=&v"(n.r[0]), "=&v"(n.r[1]), "=&v"(n.r[2]), "=&v"(n.r[3]), "=&v"(n.r[4]), "=&v"(n.r[5]), "=&v"(n.r[6]),
                 "=&v"(n.r[7]), "+v"(p.r[0]), "+v"(p.r[1]), "+v"(p.r[2]), "+v"(p.r[3]), "+v"(p.r[4]), "+v"(p.r[5]),
                 "+v"(p.r[6]), "+v"(p.r[7])
               : [p0] "v"(p0), [p1] "v"(p1), [o0] "n"(O0), [o1] "n"(O1), [o2] "n"(O2), [o3] "n"(O3));
}
// Wait until batch `p` (the last one issued) has landed.
__device__ __forceinline__ void tr4_wait(Tr4& p) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(p.r[0]), "+v"(p.r[1]), "+v"(p.r[2]), "+v"(p.r[3]), "+v"(p.r[4]), "+v"(p.r[5]), "+v"(p.r[6]),
                 "+v"(p.r[7]));
}

// Wait until at most N LDS operations issued after batch `p` are outstanding (`p` has then landed).
template <int N>
__device__ __forceinline__ void tr4_wait_n(Tr4& p) {
  asm volatile("s_waitcnt lgkmcnt(%[n])"
               : "+v"(p.r[0]), "+v"(p.r[1]), "+v"(p.r[2]), "+v"(p.r[3]), "+v"(p.r[4]), "+v"(p.r[5]), "+v"(p.r[6]),
                 "+v"(p.r[7])
               : [n] "n"(N));
}

// Two-fragment variant (four loads per batch) for kernels that are short of registers.
struct Tr2 { short4v r[4]; };
__device__ __forceinline__ bf16x8 tr2_frag(const Tr2& t, int j) {
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8v;
  short8v x = __builtin_shufflevector(t.r[2 * j], t.r[2 * j + 1], 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, x);
}
// Two fragments from two different address pairs at one byte offset (e.g. the same key step of two
// head-dim blocks, which feed two independent accumulators).
template <int O>
__device__ __forceinline__ void tr2x_issue(lds_cptr a0, lds_cptr a1, lds_cptr b0, lds_cptr b1, Tr2& n) {
  asm volatile("ds_read_b64_tr_b16 %0, %[a0] offset:%[o]\n\t"
               "ds_read_b64_tr_b16 %1, %[a1] offset:%[o]\n\t"
               "ds_read_b64_tr_b16 %2, %[b0] offset:%[o]\n\t"
               "ds_read_b64_tr_b16 %3, %[b1] offset:%[o]"
               : "=&v"(n.r[0]), "=&v"(n.r[1]), "=&v"(n.r[2]), "=&v"(n.r[3])
               : [a0] "v"(a0), [a1] "v"(a1), [b0] "v"(b0), [b1] "v"(b1), [o] "n"(O));
}

// Row-fragment batches through inline asm (same reason and same protocol as the transposed ones):
// two 16-byte fragment loads per batch, each with its own address register and byte offset.
struct R2 { bf16x8 f[2]; };
template <int O0, int O1>
__device__ __forceinline__ void r2_issue(lds_cptr a0, lds_cptr a1, R2& n) {
  asm volatile("ds_read_b128 %0, %[a0] offset:%[o0]\n\tds_read_b128 %1, %[a1] offset:%[o1]"
               : "=&v"(n.f[0]), "=&v"(n.f[1])
               : [a0] "v"(a0), [a1] "v"(a1), [o0] "n"(O0), [o1] "n"(O1));
}
template <int O0, int O1>
__device__ __forceinline__ void r2_issue_wait(lds_cptr a0, lds_cptr a1, R2& n, R2& p) {
  asm volatile("ds_read_b128 %0, %[a0] offset:%[o0]\n\tds_read_b128 %1, %[a1] offset:%[o1]\n\ts_waitcnt lgkmcnt(2)"
               : "=&v"(n.f[0]), "=&v"(n.f[1]), "+v"(p.f[0]), "+v"(p.f[1])
               : [a0] "v"(a0), [a1] "v"(a1), [o0] "n"(O0), [o1] "n"(O1));
}
__device__ __forceinline__ void r2_wait(R2& p) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(p.f[0]), "+v"(p.f[1])); }

// Four-fragment row batches.
struct R4 { bf16x8 f[4]; };

// One transposed 64-bit read of a Tr2 batch (r[0], r[1]: first fragment from the two addresses of
// the pair; r[2], r[3]: second fragment), for code that spreads the reads between other instructions.
template <int O>
__device__ __forceinline__ void tr1_issue(lds_cptr p, short4v& r) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=&v"(r) : "v"(p), "n"(O));
}

// One row fragment (for code that spreads a batch's reads between other instructions).
template <int O>
__device__ __forceinline__ void r1_issue(lds_cptr a, bf16x8& f) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(f) : "v"(a), "n"(O));
}

// Wait until at most N LDS operations issued by this wave are outstanding; `p` (a batch issued
// before those N) is then complete, and its consumers are ordered after the wait.
template <int N>
__device__ __forceinline__ void lds_wait(R4& p) {
  asm volatile("s_waitcnt lgkmcnt(%[n])" : "+v"(p.f[0]), "+v"(p.f[1]), "+v"(p.f[2]), "+v"(p.f[3]) : [n] "n"(N));
}
template <int N>
__device__ __forceinline__ void lds_wait(R2& p) {
  asm volatile("s_waitcnt lgkmcnt(%[n])" : "+v"(p.f[0]), "+v"(p.f[1]) : [n] "n"(N));
}
template <int N>
__device__ __forceinline__ void lds_wait(Tr2& p) {
  asm volatile("s_waitcnt lgkmcnt(%[n])" : "+v"(p.r[0]), "+v"(p.r[1]), "+v"(p.r[2]), "+v"(p.r[3]) : [n] "n"(N));
}

// Compile-time loop: f(IC<0>{}), ..., f(IC<N-1>{}).
template <int I> struct IC { static constexpr int value = I; constexpr operator int() const { return I; } };
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IC<I>{});
    static_for<I + 1, N>(f);
  }
}

// ---- global -> LDS staging through buffer loads -----------------------------------------------
// A TileSource addresses the rows of one head of a [T, H, D] bf16 tensor starting at row `row_base`
// through a raw buffer descriptor whose range ends with row `row_end` - 1: the hardware checks the
// whole offset (per-lane part plus scalar part) against the range and answers reads of rows from
// `row_end` on with zeros, without touching memory.  Callers put the end of what their launch
// scope may read there -- the query tile's last row for K/V, the query run's last row for Q/dO --
// so rows behind it (other units' rows, which may not have been produced yet, or the end of the
// tensor) never reach a product, and no clamping code is needed; a tile's address is a per-lane
// constant (voff) plus a wave-uniform scalar.  The bytes from row_base to row_end must stay below
// 4 GiB (checked on the host).
struct TileSource {
  __amdgpu_buffer_rsrc_t rsrc;
  int voff;        // this lane's byte offset within one pass of 256-byte lines
  int row_bytes;   // H * D * 2
};
template <int D, int NT>
__device__ __forceinline__ TileSource make_tile_source(const bf16* base, int row_base, int H, int h, int row_end, int tid) {
  TileSource s;
  const size_t first = ((size_t)row_base * H + h) * D;
  const size_t valid = ((size_t)row_end * H * D - first) * 2;
  s.rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(base + first), 0, (int)(valid > 0xFFFFFFFFull ? 0xFFFFFFFFull : valid),
                                             0x00020000);
  s.row_bytes = H * D * 2;
  const int wave = tid >> 6, lane = tid & 63, pos = lane & 15;
  const int line = wave * 4 + (lane >> 4);            // line within a pass; the swizzle repeats every pass
  int row, chunk;
  if (D == 128) {
    row = line;
    chunk = pos ^ (((row & 3) << 2) | ((row >> 2) & 3));
  } else {
    const int u = pos ^ (((line & 1) << 2) | ((line >> 1) & 3));
    row = 2 * line + (u >> 3);
    chunk = u & 7;
  }
  s.voff = row * s.row_bytes + chunk * 16;
  return s;
}
// Issues the loads for rows [row_base + row0, +ROWS) into `tile` (swizzled layout).  Completion is
// tracked by vmcnt; a barrier must follow before other waves read the tile.
template <int D, int ROWS, int NT>
__device__ __forceinline__ void stage_tile(LDS_PTR(char) tile, const TileSource& s, int row0, int tid) {
  constexpr int kLines = ROWS * D * 2 / 256, kLinesPerPass = NT / 16, kRowsPerPass = kLinesPerPass * 256 / (D * 2);
  static_assert(kLines % kLinesPerPass == 0, "tile must divide evenly over the block");
  const int wave_off = __builtin_amdgcn_readfirstlane((tid >> 6) * 1024);   // wave-uniform by construction
#pragma unroll
  for (int i = 0; i < kLines / kLinesPerPass; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(s.rsrc, tile + i * kLinesPerPass * 256 + wave_off, 16, s.voff,
                                             __builtin_amdgcn_readfirstlane((row0 + i * kRowsPerPass) * s.row_bytes), 0, 0);
}

// One pass (NT / 16 lines of 256 bytes) of stage_tile: pass i of the tile at row offset row0.
template <int D, int NT>
__device__ __forceinline__ void stage_pass(LDS_PTR(char) tile, const TileSource& s, int row0, int i, int tid) {
  constexpr int kLinesPerPass = NT / 16, kRowsPerPass = kLinesPerPass * 256 / (D * 2);
  const int wave_off = __builtin_amdgcn_readfirstlane((tid >> 6) * 1024);   // wave-uniform by construction
  const int soff = __builtin_amdgcn_readfirstlane((row0 + i * kRowsPerPass) * s.row_bytes);   // uniform as well
  __builtin_amdgcn_raw_ptr_buffer_load_lds(s.rsrc, tile + i * kLinesPerPass * 256 + wave_off, 16, s.voff, soff, 0, 0);
}

// frag_pipeline with one extra action per fragment (`side(i)`, e.g. one global->LDS load) issued
// alongside the products, so that the loads are spread over the phase instead of bunched.
template <int N, int kPre, class Load, class Use, class Side>
__device__ __forceinline__ void frag_pipeline_side(Load&& load, Use&& use, Side&& side) {
  decltype(load(0)) fr[N];
#pragma unroll
  for (int i = 0; i < N + kPre; ++i) {
    if (i < N) fr[i] = load(i);
    if (i >= kPre) {
      use(i - kPre, fr[i - kPre]);
      side(i - kPre);
    }
  }
  __builtin_amdgcn_sched_group_barrier(0x100, kPre, 0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (i + kPre < N) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
}

__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32); }

// Block -> (work item, kv head, head in group) so that the g query heads that share one K/V
// stream run back to back on the same XCD (blocks are dealt round-robin over the 8 XCDs) and
// heavy items come first on every XCD.  Returns false for padding blocks.
__device__ __forceinline__ bool map_block(int block, int g, int Hkv, int n_items, int* item, int* hk, int* hg) {
  const int xcd = block & 7, slot = block >> 3;
  *hg = slot % g;
  const int j = (slot / g) * 8 + xcd;
  if (j >= n_items * Hkv) return false;
  *item = j / Hkv;
  *hk = j % Hkv;
  return true;
}
inline int mapped_grid(int n_items, int Hkv, int g) { return ((n_items * Hkv + 7) / 8) * 8 * g; }

}  // namespace slimattn
