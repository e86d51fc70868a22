// dK/dV for bf16 inputs at head dim 128 or 64: 256 key rows per block, one wave per SIMD, 64 key rows per wave.
//
// What it computes is the dK/dV step of the backward (see bwd_bf16.hip): a block owns key rows of one
// KV head and walks every query row of the launch scope at or after them, for every query head of the
// group, in a fixed order; S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.
//
// Shape on CDNA4.  A kernel that keeps two waves per SIMD (32 keys per wave, 128 per block) is at its
// register limit at head dim 128 and reads 1.25 KB of LDS per product.  Here a block is 4 waves, one per SIMD, and a wave owns
// 64 keys (two 32-key blocks): every Q, dO, Q^T and dO^T fragment read from LDS feeds two products, the
// accumulator registers of dK^T and dV^T (256 at head dim 128) live in the accumulation half of the register file
// (they are only ever touched by products, issued from inline asm with an "a" constraint: the compiler
// cannot be told to keep a builtin product's accumulator there), and everything a vector instruction
// reads stays in the 256 architectural registers.
//
// With no second wave on the SIMD, a wave overlaps its own work, and the unit of overlap is the slot
// behind a product: the matrix unit is busy for 32 cycles per product, a product takes 4 cycles to
// issue, so about 28 cycles of other instructions (4 cycles each, an LDS read or a transcendental
// more) fit behind it for free, and whatever exceeds that, or is issued with no product running,
// costs its full time.  An iteration therefore runs
//   - 4 products that start the score accumulators S, dP of step t+1 at minus the row statistics
//     (the statistics come from the delta kernel as bf16 triples, one 16-byte load per lane and step),
//   - the 32 score products of step t+1, with one LDS row read (for two head-dim steps ahead) and one
//     piece of bookkeeping behind each: the walk to step t+2, the loads that stage its Q/dO tiles and
//     statistics, its masks, the moves of the fragment addresses to the next LDS stage, the first
//     transposed reads of the gradient phase,
//   - the 32 gradient products of step t, with one transposed LDS read and one slot of the element-
//     wise work of step t+1 (exp2, dS, packing to bf16) behind each,
//   - one barrier.
// Query steps are 32 rows; their tiles are staged two steps ahead through three LDS stages; the
// block's 256 V rows stay in LDS, its K fragments in registers.
//
// Hazards of the inline-asm products (the compiler does not know what they are and adds no wait
// states): their results are read only by later products on the same accumulator (at least three
// other products in between) and, after the loop or in the masked path, behind explicit wait states;
// their B operands were packed by vector instructions a whole phase earlier, except the zero
// fragments of the first step (see mfma_acc).
#include <hip/hip_runtime.h>

#include "internal.h"
#include "mfma_utils.h"

namespace slimattn {
namespace {

constexpr int kKeys = 256;                              // key rows per block: 4 waves x 64
constexpr int kQStep = 32;
constexpr int kStages = 3;
template <int D> constexpr int kNKS = D / 16;           // head-dim steps of a score product
template <int D> constexpr int kNDB = D / 32;           // head-dim blocks of a gradient accumulator
template <int D> constexpr int kRowBytes = D * 2;
template <int D> constexpr int kTileBytes = kQStep * kRowBytes<D>;   // one Q or dO tile
template <int D> constexpr int kStageBytes = 2 * kTileBytes<D>;      // [Q tile, dO tile]
template <int D> constexpr int kVBase = kStages * kStageBytes<D>;
template <int D> constexpr int kVBytes = kKeys * kRowBytes<D>;
template <int D> constexpr int kGradBatches = 2 * kNDB<D>;           // batches of transposed reads in the gradient phase
constexpr float kLog2e = 1.4426950408889634f;

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned uintx4;   // a packed bf16x8 fragment, by dword
__device__ __forceinline__ bf16x8 as_frag(uintx4 x) { return __builtin_bit_cast(bf16x8, x); }

// START: the product starts its accumulator (C = 0) instead of adding to it.  The accumulators are never
// initialised by compiler-generated moves, and a START product waits a few cycles before it issues: the
// compiler does not know that the asm is a matrix product, so it separates neither such a move nor a
// vector write of an operand register (the zero fragments of the first step are written right in front
// of the first product) from it by the wait states the hardware needs.  The other products read only
// registers written a whole phase earlier (packed P, dS) or by waited-for LDS reads.
template <bool START>
__device__ __forceinline__ void mfma_acc(floatx16& acc, bf16x8 a, bf16x8 b) {
  if (START) asm volatile("s_nop 7\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(acc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// Score products of one step: s[kb] = Q K_kb^T - lse (log2 units, kf holds k * scale * log2 e),
// dp[kb] = dO V_kb^T - delta, for the wave's two key blocks.  pq[] point at the step's Q tile (the dO
// tile follows it), v_rel is the byte distance from there to this wave's V rows.  The accumulators
// start at minus the row statistics: `stat` holds, for the lane's row (l32), -lse2 and -delta as three
// bf16 terms each ({l, l, l, 0, d, d, d, 0}; the terms of a triple add up to the fp32 value), and a
// product with a fragment of ones (ones_l picks the first triple, ones_d the second; zero in the upper
// half-wave, whose copy of `stat` therefore does not count) puts their sums into every column of the
// row.  That costs four products and no vector or LDS instruction, where loading the 64 accumulator
// registers costs a quarter of the phase.  In `masked` steps the scores of pairs that do not count
// (local row - 4*half outside [rel_lo[kb], rel_hi): before the lane's key, or past the end of the query
// run) are then set to -inf, so that their probability and dS come out as zero.
// One batch of LDS reads per head-dim step: the Q and dO fragments and the two V fragments.
template <int D, class Between>
__device__ __forceinline__ void score_products(const lds_cptr (&pq)[kNKS<D>], int v_rel, bf16x8 stat, uintx4 ones_l, uintx4 ones_d,
                                               const bf16x8 (&kf)[2][kNKS<D>], floatx16 (&s)[2], floatx16 (&dp)[2],
                                               bool masked, const int (&rel_lo)[2], int rel_hi, Between&& between) {
  // Fragment i of head-dim step u: 0 Q rows, 1 dO rows, 2/3 the V rows of the two key blocks.  The
  // reads of step u + 2 are issued one behind each product of step u (an LDS read takes about twice the
  // issue time of a plain instruction: four in a row would outlast the product they follow); those of
  // the first two steps run while the accumulators are started.
  R4 g[kNKS<D>];
  lds_cptr pv = pq[0];
  auto issue_one = [&](auto uc, auto ic) {
    constexpr int u = decltype(uc)::value, i = decltype(ic)::value;
    if constexpr (i == 0) r1_issue<0>(pq[u], g[u].f[0]);
    if constexpr (i == 1) { r1_issue<kTileBytes<D>>(pq[u], g[u].f[1]); pv = pq[u] + v_rel; }
    if constexpr (i == 2) r1_issue<0>(pv, g[u].f[2]);
    if constexpr (i == 3) r1_issue<32 * kRowBytes<D>>(pv, g[u].f[3]);
  };
  static_for<0, 4>([&](auto ic) { issue_one(IC<0>{}, ic); });
  // asm: two of the four products are equal and the compiler would compute them once and copy
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(s[0]) : "v"(stat), "v"(ones_l));
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(s[1]) : "v"(stat), "v"(ones_l));
  static_for<0, 4>([&](auto ic) { issue_one(IC<1>{}, ic); });
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(dp[0]) : "v"(stat), "v"(ones_d));
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(dp[1]) : "v"(stat), "v"(ones_d));
  if (__builtin_expect(masked, 0)) {
    // the products above are asm statements: the compiler does not separate them from readers of
    // their results by the wait states the hardware needs
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(s[0]), "+v"(s[1]));
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const unsigned span = (unsigned)max(rel_hi - rel_lo[kb], 0);   // c - rel_lo in [0, span) <=> the pair counts
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int c = 8 * (r >> 2) + (r & 3);           // c + 4*half = local row
        s[kb][r] = (unsigned)(c - rel_lo[kb]) < span ? s[kb][r] : -INFINITY;
      }
    }
  }
  static_for<0, kNKS<D>>([&](auto uc) {
    constexpr int u = decltype(uc)::value;
    constexpr bool more = u + 2 < kNKS<D>;
    lds_wait<4>(g[u]);                                  // behind step u: step u + 1 or, at the end, a batch of gradient reads
    s[0] = mfma32(g[u].f[0], kf[0][u], s[0]);
    if constexpr (more) issue_one(IC<u + 2>{}, IC<0>{});
    between(IC<4 * u + 0>{});
    __builtin_amdgcn_sched_barrier(0);
    s[1] = mfma32(g[u].f[0], kf[1][u], s[1]);
    if constexpr (more) issue_one(IC<u + 2>{}, IC<1>{});
    between(IC<4 * u + 1>{});
    __builtin_amdgcn_sched_barrier(0);
    dp[0] = mfma32(g[u].f[1], g[u].f[2], dp[0]);
    if constexpr (more) issue_one(IC<u + 2>{}, IC<2>{});
    between(IC<4 * u + 2>{});
    __builtin_amdgcn_sched_barrier(0);
    dp[1] = mfma32(g[u].f[1], g[u].f[3], dp[1]);
    if constexpr (more) issue_one(IC<u + 2>{}, IC<3>{});
    between(IC<4 * u + 3>{});
    __builtin_amdgcn_sched_barrier(0);
  });
}

// Element-wise work, P = exp2(S - lse) and dS = P (dP - delta), as a stream of 32 values cut into slots,
// one slot behind each gradient product (two at head dim 64).  Slot j: the exponential of value j, the dS
// product of value j - 1, and one packing to bf16: P of the pair (j - 1, j) in odd slots, dS of the pair
// (j - 2, j - 1) in even ones; the last slot also finishes value 31.  One transcendental and two plain
// vector instructions: with the product's own issue that fills, and does not exceed, the time the matrix
// unit spends on one product.  Each slot is one asm statement: the compiler keeps asm statements in
// program order (as ordinary code it moves the whole stream behind the last product of the loop body,
// where nothing overlaps it) and puts no wait states between the instructions.  A transcendental
// result may not be read by the very next vector instruction: the instruction behind each
// exponential reads other registers.
// Order of the values: the first half of the stream (which runs behind the products of the first 16-row
// half) holds registers 8..15 of the two key blocks, i.e. the packed fragments of the second 16-row half,
// which go to the temporaries tp, td; the second half holds registers 0..7, whose fragments go straight
// into pf[.][0], ds[.][0]: those were last read by the products of the first half.  Only the
// temporaries are copied at the end of the iteration.
struct EwValue { int kb, r; };
constexpr EwValue ew_value(int j) { return j < 16 ? EwValue{j >> 3, 8 + (j & 7)} : EwValue{(j - 16) >> 3, (j - 16) & 7}; }
template <int J>
__device__ __forceinline__ void ew_slot(floatx16 (&s)[2], floatx16 (&dp)[2], uintx4 (&pf)[2][2], uintx4 (&ds)[2][2],
                                        uintx4 (&tp)[2], uintx4 (&td)[2]) {
  constexpr EwValue v0 = ew_value(J), v1 = ew_value(J > 0 ? J - 1 : 0), v2 = ew_value(J > 1 ? J - 2 : 0);
  auto put_p = [&](EwValue v, unsigned w) {             // the word of the pair that ends at value v
    if (v.r >= 8) tp[v.kb][(v.r & 7) >> 1] = w; else pf[v.kb][0][(v.r & 7) >> 1] = w;
  };
  auto put_ds = [&](EwValue v, unsigned w) {
    if (v.r >= 8) td[v.kb][(v.r & 7) >> 1] = w; else ds[v.kb][0][(v.r & 7) >> 1] = w;
  };
  float e = s[v0.kb][v0.r];
  if constexpr (J == 0) {
    asm volatile("v_exp_f32 %0, %0" : "+v"(e));
    s[v0.kb][v0.r] = e;
  } else if constexpr (J & 1) {
    float m = dp[v1.kb][v1.r];
    unsigned w;
    asm volatile("v_exp_f32 %0, %0\n\tv_mul_f32 %1, %3, %1\n\tv_cvt_pk_bf16_f32 %2, %3, %0"
                 : "+v"(e), "+v"(m), "=&v"(w) : "v"(s[v1.kb][v1.r]));
    s[v0.kb][v0.r] = e;
    dp[v1.kb][v1.r] = m;
    put_p(v0, w);
    if constexpr (J == 31) {
      float m2 = dp[v0.kb][v0.r];
      unsigned w2;
      asm volatile("v_mul_f32 %0, %2, %0\n\tv_cvt_pk_bf16_f32 %1, %3, %0" : "+v"(m2), "=&v"(w2) : "v"(e), "v"(dp[v1.kb][v1.r]));
      dp[v0.kb][v0.r] = m2;
      put_ds(v0, w2);
    }
  } else {
    float m = dp[v1.kb][v1.r];
    unsigned w;
    asm volatile("v_exp_f32 %0, %0\n\tv_mul_f32 %1, %3, %1\n\tv_cvt_pk_bf16_f32 %2, %4, %1"
                 : "+v"(e), "+v"(m), "=&v"(w) : "v"(s[v1.kb][v1.r]), "v"(dp[v2.kb][v2.r]));
    s[v0.kb][v0.r] = e;
    dp[v1.kb][v1.r] = m;
    put_ds(v1, w);
  }
}

// Read i (of four) of gradient batch B: the dO^T fragment (reads 0, 1) and the Q^T fragment (2, 3) of
// head-dim block B % 4, rows 16 (B / 4) .. +16 of the step's tiles.
template <int D, int B, int I>
__device__ __forceinline__ void grad_read(const lds_cptr (&pqt)[kNDB<D>][2], Tr2 (&tb)[kGradBatches<D>]) {
  constexpr int st = B / kNDB<D>, db = B % kNDB<D>;
  tr1_issue<st * 16 * kRowBytes<D> + (I < 2 ? kTileBytes<D> : 0)>(pqt[db][I & 1], tb[B].r[I]);
}

// Gradient products of one step, dV_kb^T += dO^T P_kb and dK_kb^T += Q^T dS_kb, with P, dS packed in
// pf[kb][half16], ds[kb][half16]; pqt[][] point at the step's Q tile.  Per head-dim block and 16-row half
// one batch of two transposed fragments (dO^T, Q^T), each feeding both key blocks.  The element-wise work
// of the next step (its scores in s, dp) is spread between the products (see ew_slot), and its packed
// results are left in pf[.][0], ds[.][0] (first 16-row half) and tp, td (second half).  FIRST: the block's first call, which starts the accumulators.
template <int D, bool FIRST>
__device__ __forceinline__ void gradient_products(const lds_cptr (&pqt)[kNDB<D>][2], uintx4 (&pf)[2][2], uintx4 (&ds)[2][2],
                                                  floatx16 (&dk)[2][kNDB<D>], floatx16 (&dv)[2][kNDB<D>], floatx16 (&s)[2],
                                                  floatx16 (&dp)[2], uintx4 (&tp)[2], uintx4 (&td)[2],
                                                  Tr2 (&tb)[kGradBatches<D>]) {
  // batch b: head-dim block b % 4 of 16-row half b / 4 (first half first: its P, dS die early); its
  // four reads are issued one behind each product of batch b - 2, those of batches 0 and 1 behind the
  // last score products (by the caller)
  constexpr int kPer = 32 / (4 * kGradBatches<D>);       // element-wise values per product slot (1 at d 128, 2 at d 64)
  auto ew = [&](auto qc) {                              // the element-wise work behind product q of the phase
    constexpr int q = decltype(qc)::value;
    static_for<0, kPer>([&](auto ec) { ew_slot<kPer * q + decltype(ec)::value>(s, dp, pf, ds, tp, td); });
  };
  static_for<0, kGradBatches<D>>([&](auto ic) {
    constexpr int b = decltype(ic)::value, st = b / kNDB<D>, db = b % kNDB<D>;
    constexpr bool more = b + 2 < kGradBatches<D>;
    lds_wait<(b + 1 < kGradBatches<D>) ? 4 : 0>(tb[b]);
    constexpr bool kStart = FIRST && st == 0;
    mfma_acc<kStart>(dv[0][db], tr2_frag(tb[b], 0), as_frag(pf[0][st]));
    if constexpr (more) grad_read<D, b + 2, 0>(pqt, tb);
    ew(IC<4 * b + 0>{});
    __builtin_amdgcn_sched_barrier(0);
    mfma_acc<kStart>(dv[1][db], tr2_frag(tb[b], 0), as_frag(pf[1][st]));
    if constexpr (more) grad_read<D, b + 2, 1>(pqt, tb);
    ew(IC<4 * b + 1>{});
    __builtin_amdgcn_sched_barrier(0);
    mfma_acc<kStart>(dk[0][db], tr2_frag(tb[b], 1), as_frag(ds[0][st]));
    if constexpr (more) grad_read<D, b + 2, 2>(pqt, tb);
    ew(IC<4 * b + 2>{});
    __builtin_amdgcn_sched_barrier(0);
    mfma_acc<kStart>(dk[1][db], tr2_frag(tb[b], 1), as_frag(ds[1][st]));
    if constexpr (more) grad_read<D, b + 2, 3>(pqt, tb);
    ew(IC<4 * b + 3>{});
    __builtin_amdgcn_sched_barrier(0);
  });
}

// p += d as an asm statement: stays in the slot where it is written (the compiler gathers plain
// additions of this kind in one place, where they outlast the product they should hide behind).
__device__ __forceinline__ void lds_ptr_add(lds_cptr& p, int d) {
  unsigned x = (unsigned)(size_t)p;
  asm volatile("v_add_u32 %0, %1, %0" : "+v"(x) : "s"(d));
  p = (lds_cptr)(size_t)x;
}

struct Step { int i0, hi, head; };                      // rows [i0, min(i0 + 32, hi)) of one query head

template <int D>
__device__ __forceinline__ void dkdv_wide_block(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v, const bf16* __restrict__ dO,
    const bf16x8* __restrict__ stat3, float* __restrict__ acc_dk, float* __restrict__ acc_dv,
    bf16* __restrict__ dK, bf16* __restrict__ dV, const KvItem* __restrict__ items, int n_items, const Seg* __restrict__ segs,
    int T, int Hq, int Hkv, float scale, float* __restrict__ parts) {
  __shared__ __attribute__((aligned(1024))) char smem[kVBase<D> + kVBytes<D>];   // three [Q, dO] stages, then the V tile

  const int g = Hq / Hkv;
  const int item_idx = blockIdx.x / Hkv, hk = blockIdx.x % Hkv;
  if (item_idx >= n_items) return;
  const KvItem it = items[item_idx];
  // where the rows' sums come from and go to: rows below load_until continue the partial sum an earlier unit left in
  // the fp32 accumulators; rows from final_from on get no later contribution and are written as dK/dV in the
  // output type, the others into the accumulators
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int kv0w = it.kv_row0 + 64 * wave, kv_end = it.kv_row0 + it.kv_rows;
  LDS_PTR(char) lds = (LDS_PTR(char))smem;

  // Flattened walk (block-uniform): runs from the last to the first, inside a run steps of 32 rows from
  // the top down, inside a step the heads of the group.
  int sgi = it.seg_end - 1, hh = 0;
  Seg sg = segs[sgi];
  int lo = max(sg.q_lo, it.kv_row0);
  int n = (sg.q_hi - lo + kQStep - 1) / kQStep - 1;
  bool more = true;                                     // the walk has a step that was not handed out yet
  // The next step of the walk, in three pieces (the loop runs each behind a different product; between
  // pieces the values are pinned with empty asm statements so that the compiler leaves the arithmetic
  // where it is written).  A step is only taken when `more`; otherwise d keeps its value.
  auto next_step_a = [&](Step& d) -> bool {            // the step's coordinates
    const bool ok = more;
    d.i0 = __builtin_amdgcn_readfirstlane(ok ? lo + n * kQStep : d.i0);   // (block-uniform anyway: tells the compiler)
    d.hi = __builtin_amdgcn_readfirstlane(ok ? sg.q_hi : d.hi);
    d.head = __builtin_amdgcn_readfirstlane(ok ? hk * g + hh : d.head);
    asm volatile("" : "+s"(d.i0), "+s"(d.hi), "+s"(d.head));
    return ok;
  };
  auto next_step_b = [&](bool ok) {                     // move on: next head, or next 32 rows down
    const bool wrap = ok && hh + 1 == g;
    hh = !ok ? hh : wrap ? 0 : hh + 1;
    n -= wrap ? 1 : 0;
  };
  auto next_step_c = [&](bool ok) {                     // the run is used up: the one before it, if any
    if (__builtin_expect((int)ok & (int)(n < 0), 0)) {
      if (--sgi < it.seg_begin) {
        more = false;
      } else {
        sg = segs[sgi];
        lo = max(sg.q_lo, it.kv_row0);
        n = (sg.q_hi - lo + kQStep - 1) / kQStep - 1;
      }
    }
  };
  auto next_step = [&](Step& d) -> bool {
    const bool ok = next_step_a(d);
    next_step_b(ok);
    next_step_c(ok);
    return ok;
  };

  // Q and dO rows come through descriptors based at the tile's first key row (head 0) whose range ends with the
  // query run of the step being staged: the rows of a step that lie past the end of its run (they belong to
  // another unit, whose dO may not exist yet, or to the next sample) read as zeros and add nothing to the
  // gradient products, whatever the memory holds.
  const bf16* const q_base = q + (size_t)it.kv_row0 * Hq * D;
  const bf16* const do_base = dO + (size_t)it.kv_row0 * Hq * D;
  auto run_range = [&](const Step& d) -> int { return (d.hi - it.kv_row0) * (Hq * kRowBytes<D>); };   // bytes up to the run's end
  auto rsrc_of = [&](const bf16* base, int bytes) -> __amdgpu_buffer_rsrc_t {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, bytes, 0x00020000);
  };
  const TileSource srcQ = make_tile_source<D, 256>(q, it.kv_row0, Hq, 0, T, tid);    // (voff, row_bytes; its range is replaced per step)
  auto stage = [&](const Step& d, int st) {             // a step's Q and dO tiles straight into LDS
    TileSource a = srcQ, b = srcQ;
    a.rsrc = rsrc_of(q_base, run_range(d));
    b.rsrc = rsrc_of(do_base, run_range(d));
    a.voff += d.head * kRowBytes<D>;
    b.voff += d.head * kRowBytes<D>;
    stage_tile<D, kQStep, 256>(lds + st * kStageBytes<D>, a, d.i0 - it.kv_row0, tid);
    stage_tile<D, kQStep, 256>(lds + st * kStageBytes<D> + kTileBytes<D>, b, d.i0 - it.kv_row0, tid);
  };
  // A step's statistics for this lane's row (-lse2, -delta as bf16 triples; rows past the end of the run
  // are masked later), through a buffer descriptor: a per-lane byte offset (stat_voff) plus a scalar one.
  const __amdgpu_buffer_rsrc_t stat_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)stat3, 0, (int)((size_t)T * Hq * 16), 0x00020000);
  // (a row past the end of the run takes the run's last row: finite numbers of this launch's own scope,
  // whatever the rest of the array holds; its scores are masked)
  auto stat_voff = [&](const Step& d) -> int { return min(d.i0 + l32, d.hi - 1) * 16; };
  auto load_stat_at = [&](const Step& d, int voff) -> bf16x8 {
    return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(stat_rsrc, voff, d.head * T * 16, 0));
  };
  auto load_stat = [&](const Step& d) -> bf16x8 { return load_stat_at(d, stat_voff(d)); };

  Step d_s, d_n;                                        // the step whose scores come next, the step to stage
  next_step(d_s);                                       // a key tile always has at least its own rows
  d_n = d_s;
  stage(d_s, 0);
  bf16x8 stat_s = load_stat(d_s), stat_n = stat_s;
  const unsigned one2 = half ? 0u : 0x3F803F80u, one1 = half ? 0u : 0x00003F80u;   // bf16 {1, 1}, {1, 0}; lower half-wave only
  const uintx4 ones_l = {one2, one1, 0u, 0u}, ones_d = {0u, 0u, one2, one1};
  bool have_s = true;
  {
    const TileSource srcV = make_tile_source<D, 256>(v, it.kv_row0, Hkv, hk, kv_end, tid);
    stage_tile<D, kKeys, 256>(lds + kVBase<D>, srcV, 0, tid);
  }
  bf16x8 kf[2][kNKS<D>];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const size_t off = ((size_t)min(kv0w + 32 * kb + l32, T - 1) * Hkv + hk) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < kNKS<D>; ++ks) {
      kf[kb][ks] = scale8(*reinterpret_cast<const bf16x8*>(k + off + 16 * ks), scale * kLog2e);
      __builtin_amdgcn_sched_barrier(0);              // one fragment at a time: this set-up code must not need many registers
    }
  }
  // pq[]: row-fragment addresses in the stage of the step whose scores are computed next; pqt[][]:
  // transposed-fragment addresses in the stage of the step whose gradients are computed next.  Both move
  // one stage per iteration (with wrap-around), so every LDS offset in the products is an immediate.
  lds_cptr pq[kNKS<D>], pqt[kNDB<D>][2];
#pragma unroll
  for (int ks = 0; ks < kNKS<D>; ++ks) pq[ks] = lds_row_ptr<D>(lds, l32, 16 * ks + 8 * half);
#pragma unroll
  for (int db = 0; db < kNDB<D>; ++db) lds_tr_ptrs<D>(lds, 32 * db, lane, pqt[db][0], pqt[db][1]);
  int v_rel = kVBase<D> + wave * 64 * kRowBytes<D>;           // the swizzle of row 64 w + 32 kb + l32 equals that of row l32
  floatx16 dk[2][kNDB<D>], dv[2][kNDB<D>];                    // started by the first iteration's products
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  // Masks of a step for this wave: local rows [rel_lo0 (+32 for the second key block), rel_hi) minus 4*half
  // count (from the lane's key on, up to the end of the query run); `masked` (wave-uniform): the step has a
  // row before the wave's last key or past the end of its run.  One flag, one branch per step: branches,
  // taken or not, are among the most expensive instructions of this loop.
  struct Mask { int rel_lo0, rel_hi; bool masked; };
  auto masks = [&](const Step& d) -> Mask {
    return Mask{kv0w + l32 - d.i0 - 4 * half, d.hi - d.i0 - 4 * half, d.i0 < kv0w + 63 || d.i0 + kQStep > d.hi};
  };
  Mask m_s = masks(d_s), m_n = m_s;
  const int wave_off = __builtin_amdgcn_readfirstlane((tid >> 6) * 1024);   // this wave's lines within a staging pass

  // One loop body for everything.  Iteration: score products of step d_s (tiles in stage st_s, where pq
  // points); gradient products of the step before it (tiles in the stage where pqt points; its P, dS in
  // pf, ds) with the element-wise work of d_s spread between them.  Each wave is alone on its SIMD, so
  // every instruction that is not issued while a product runs costs its full issue time: the walk to
  // the step after next, the loads that stage it into st_n, its masks and the moves of the fragment
  // addresses are cut into pieces of a few instructions, one piece behind each score product (the
  // element-wise work fills the slots behind the gradient products).  The first iteration has no step
  // before: pf, ds are zero and pqt points at stage 0 (finite numbers times zero).  The last iteration
  // has no d_s: scores and element-wise work run on the stale tile of stage st_s and nobody uses them.
  // Stage st_n's last readers (the gradient products two iterations back) finished before the barrier
  // that ended the previous iteration.
  uintx4 pf[2][2], ds[2][2];                            // packed P, dS of the step whose gradient products come next
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) { pf[kb][h2] = uintx4{0u, 0u, 0u, 0u}; ds[kb][h2] = uintx4{0u, 0u, 0u, 0u}; }
  int st_s = 0;
  int dt_pend = 0;                                      // pqt's move to the stage scored last, applied in the next score phase
  bool again;
  auto iteration = [&](auto first_c) {
    constexpr bool first = decltype(first_c)::value != 0;
    const int st_n = st_s == 2 ? 0 : st_s + 1;
    const int dq_ = st_s == 2 ? -2 * kStageBytes<D> : kStageBytes<D>;   // pq's move to the next stage
    bool have_n = false;
    int voff_n = 0, soff_n = 0;
    Tr2 tb[kGradBatches<D>];                               // the gradient phase's batches of transposed fragments
    const int m0_n = st_n * kStageBytes<D> + wave_off;     // where this wave's lines of the first pass go
    // slots of the pieces (behind score product k): spread out at d 128 (32 slots), packed at d 64 (16).
    // A piece is a handful of instructions: what does not fit behind its product delays the next one.
    constexpr int kSlotWalkA = D == 128 ? 4 : 2, kSlotWalkB = D == 128 ? 5 : 3, kSlotWalkC = D == 128 ? 6 : 3;
    constexpr int kSlotStatA = D == 128 ? 7 : 4, kSlotStat = D == 128 ? 8 : 5, kSlotAddr = D == 128 ? 9 : 4;
    constexpr int kSlotLoad = D == 128 ? 10 : 6, kLoadStride = D == 128 ? 2 : 1, kSlotMask = D == 128 ? 18 : 7;
    constexpr int kSlotGrad = 4 * (kNKS<D> - 2);
    constexpr int kPasses = kTileBytes<D> / 4096;         // staging loads per tile (256 threads x 16 bytes each)
    bool ok_n = false;
    int stat_off = 0, range_n = 0;
    auto between = [&](auto kc) {                       // piece k of the bookkeeping, behind score product k
      constexpr int k = decltype(kc)::value;
      if constexpr (k < kNDB<D>) { lds_ptr_add(pqt[k][0], dt_pend); lds_ptr_add(pqt[k][1], dt_pend); }
      if constexpr (k == kSlotWalkA) { ok_n = next_step_a(d_n); have_n = have_s && ok_n; }
      if constexpr (k == kSlotWalkB) next_step_b(ok_n);
      if constexpr (k == kSlotWalkC) next_step_c(ok_n);
      if constexpr (k == kSlotStatA) { stat_off = stat_voff(d_n); asm volatile("" : "+v"(stat_off)); }
      if constexpr (k == kSlotStat) stat_n = load_stat_at(d_n, stat_off);   // d_n always names a real step (the last one, when the walk has ended)
      if constexpr (k == kSlotAddr) {
        voff_n = srcQ.voff + d_n.head * kRowBytes<D>;   // the Q and dO sources differ in their descriptors only
        soff_n = __builtin_amdgcn_readfirstlane((d_n.i0 - it.kv_row0) * srcQ.row_bytes);
        range_n = __builtin_amdgcn_readfirstlane(run_range(d_n));
        asm volatile("" : "+v"(voff_n), "+s"(soff_n), "+s"(range_n));
      }
      if constexpr (k >= kSlotLoad && k < kSlotLoad + 2 * kPasses * kLoadStride && (k - kSlotLoad) % kLoadStride == 0) {
        // one load each: the passes of the Q tile, then of the dO tile
        constexpr int x = (k - kSlotLoad) / kLoadStride, tile = x / kPasses, pass = x % kPasses;
        constexpr int kRowsPerPass = 4096 / kRowBytes<D>;
        // (when the walk has ended d_n still names the last step: its tile is staged once more, into a stage nobody reads)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_of(tile ? do_base : q_base, range_n), lds + m0_n + tile * kTileBytes<D> + pass * 4096, 16,
                                                 voff_n, soff_n + pass * kRowsPerPass * srcQ.row_bytes, 0, 0);
      }
      if constexpr (k == kSlotMask) m_n = masks(d_n);
      if constexpr (k >= kSlotGrad && k < kSlotGrad + 8) {   // the gradient phase's first two batches of reads
        grad_read<D, (k - kSlotGrad) / 4, (k - kSlotGrad) % 4>(pqt, tb);
        if constexpr (k - kSlotGrad < kNKS<D>) lds_ptr_add(pq[k - kSlotGrad], dq_);
      }
      if constexpr (k == kSlotGrad + 7) v_rel -= dq_;
    };
    floatx16 s[2], dp[2];
    uintx4 tp[2], td[2];                                // packed P, dS of the second 16-row half of the step being scored
    const int rel_lo[2] = {m_s.rel_lo0, m_s.rel_lo0 + 32};
    score_products<D>(pq, v_rel, stat_s, ones_l, ones_d, kf, s, dp, m_s.masked, rel_lo, m_s.rel_hi, between);
    gradient_products<D, first>(pqt, pf, ds, dk, dv, s, dp, tp, td, tb);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) { pf[kb][1] = tp[kb]; ds[kb][1] = td[kb]; }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    again = have_s;
    d_s = d_n;
    m_s = m_n;
    stat_s = stat_n;
    have_s = have_n;
    dt_pend = first ? 0 : (st_s == 0 ? -2 * kStageBytes<D> : kStageBytes<D>);   // pqt moves to the stage just scored
    st_s = st_n;
  };
  iteration(IC<1>{});
  while (again) iteration(IC<0>{});
  // the last products' results must have landed before any vector instruction reads them (the
  // compiler does not know that the asm statements are matrix products): explicit wait states
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15");

  if (it.slot < 0 && it.final_from <= it.kv_row0 && it.load_until <= it.kv_row0) {
    // The fused launch's case: bf16 rows of dK, then of dV, out through LDS (stages and V tile are free behind
    // the loop's last barrier; each wave uses a part of its own).  A lane owns a row's values in pieces of 4
    // columns, and written as they stand each store instruction would touch 32 rows with 16 bytes each;
    // transposed, a store instruction writes whole rows.
    constexpr int kOutStride = kRowBytes<D> + 16, kChunks = kRowBytes<D> / 16, kRowsPerStore = 64 / kChunks;
    static_assert(4 * 64 * kOutStride <= kVBase<D> + kVBytes<D>, "the transposition areas must fit the block's LDS");
    LDS_PTR(char) ep = lds + wave * 64 * kOutStride;
    const int st_row = lane / kChunks, st_chunk = lane % kChunks;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int db = 0; db < kNDB<D>; ++db)
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            bf16x4 w;
#pragma unroll
            for (int x = 0; x < 4; ++x) w[x] = which ? (bf16)dv[kb][db][4 * gq + x] : (bf16)(dk[kb][db][4 * gq + x] * scale);
            *reinterpret_cast<LDS_PTR(bf16x4)>(ep + (32 * kb + l32) * kOutStride + (32 * db + 8 * gq + 4 * half) * 2) = w;
          }
      bf16* out = which ? dV : dK;
#pragma unroll
      for (int j = 0; j < 64 / kRowsPerStore; ++j) {
        const int r = j * kRowsPerStore + st_row;
        const bf16x8 w = *reinterpret_cast<LDS_PTR(const bf16x8)>(ep + r * kOutStride + st_chunk * 16);
        if (kv0w + r < kv_end) *reinterpret_cast<bf16x8*>(out + ((size_t)(kv0w + r) * Hkv + hk) * D + st_chunk * 8) = w;
      }
    }
    return;
  }
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const int my_key = kv0w + 32 * kb + l32;
    if (it.slot >= 0) {
      // one part of a divided key tile: fp32 partial tile [slot][kv head][dK, dV][256 rows][D]
      float* pk_ = parts + ((size_t)it.slot * Hkv + hk) * (2 * kKeys * D) + (size_t)(64 * wave + 32 * kb + l32) * D;
      float* pv_ = pk_ + kKeys * D;
#pragma unroll
      for (int db = 0; db < kNDB<D>; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int off = 32 * db + 8 * gq + 4 * half;
          floatx4 a, b;
#pragma unroll
          for (int x = 0; x < 4; ++x) { a[x] = dk[kb][db][4 * gq + x] * scale; b[x] = dv[kb][db][4 * gq + x]; }
          *reinterpret_cast<floatx4*>(pk_ + off) = a;
          *reinterpret_cast<floatx4*>(pv_ + off) = b;
        }
    } else if (my_key < kv_end) {
      const size_t base = ((size_t)my_key * Hkv + hk) * D;
      const bool load_acc = my_key < it.load_until, store_final = my_key >= it.final_from;
#pragma unroll
      for (int db = 0; db < kNDB<D>; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const size_t off = base + 32 * db + 8 * gq + 4 * half;
          floatx4 a, b;
#pragma unroll
          for (int x = 0; x < 4; ++x) { a[x] = dk[kb][db][4 * gq + x] * scale; b[x] = dv[kb][db][4 * gq + x]; }
          if (load_acc) {
            a += *reinterpret_cast<const floatx4*>(acc_dk + off);
            b += *reinterpret_cast<const floatx4*>(acc_dv + off);
          }
          if (store_final) {
            bf16x4 wa, wb;
#pragma unroll
            for (int x = 0; x < 4; ++x) { wa[x] = (bf16)a[x]; wb[x] = (bf16)b[x]; }
            *reinterpret_cast<bf16x4*>(dK + off) = wa;
            *reinterpret_cast<bf16x4*>(dV + off) = wb;
          } else {
            *reinterpret_cast<floatx4*>(acc_dk + off) = a;
            *reinterpret_cast<floatx4*>(acc_dv + off) = b;
          }
        }
    }
  }
}

// One kernel per head dim (plain functions: the launch below names them).
__global__ __launch_bounds__(256, 1) void dkdv_wide_bf16_kernel_d128(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v, const bf16* __restrict__ dO,
    const bf16x8* __restrict__ stat3, float* __restrict__ acc_dk, float* __restrict__ acc_dv, bf16* __restrict__ dK,
    bf16* __restrict__ dV, const KvItem* __restrict__ items, int n_items, const Seg* __restrict__ segs, int T, int Hq, int Hkv,
    float scale, float* __restrict__ parts) {
  dkdv_wide_block<128>(q, k, v, dO, stat3, acc_dk, acc_dv, dK, dV, items, n_items, segs, T, Hq, Hkv, scale, parts);
}
__global__ __launch_bounds__(256, 1) void dkdv_wide_bf16_kernel_d64(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v, const bf16* __restrict__ dO,
    const bf16x8* __restrict__ stat3, float* __restrict__ acc_dk, float* __restrict__ acc_dv, bf16* __restrict__ dK,
    bf16* __restrict__ dV, const KvItem* __restrict__ items, int n_items, const Seg* __restrict__ segs, int T, int Hq, int Hkv,
    float scale, float* __restrict__ parts) {
  dkdv_wide_block<64>(q, k, v, dO, stat3, acc_dk, acc_dv, dK, dV, items, n_items, segs, T, Hq, Hkv, scale, parts);
}

}  // namespace

int launch_bwd_dkdv_wide_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, const void* dO, const void* stat3,
                            float* acc_dk, float* acc_dv, void* dK, void* dV, const KvItem* items, int n_items, const Seg* segs,
                            float* parts) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const dim3 grid((unsigned)(n_items * p.n_kv_heads)), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(dkdv_wide_bf16_kernel_d128, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, (const bf16x8*)stat3, acc_dk, acc_dv, (bf16*)dK, (bf16*)dV, items, n_items,
                       segs, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale, parts);
  else
    hipLaunchKernelGGL(dkdv_wide_bf16_kernel_d64, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, (const bf16x8*)stat3, acc_dk, acc_dv, (bf16*)dK, (bf16*)dV, items, n_items,
                       segs, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale, parts);
  return (int)hipGetLastError();
}

}  // namespace slimattn
