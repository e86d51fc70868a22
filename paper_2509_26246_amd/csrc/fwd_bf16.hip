// Forward, bf16 inputs, MFMA products with fp32 accumulation, fp32 online softmax: the kernels with two waves
// per SIMD (head dim 64, and odd numbers of query heads per KV head; even groups at head dim 128 run the
// one-wave kernel of fwd_wide_bf16.hip).
//
// What it computes (paper: PackFlow section -- a slice's queries attend to the cached keys and
// values of every earlier slice of the sample and causally to the slice itself): for a query tile
// of 128 rows of one head, walk the sample's keys kv_start .. last row in tiles of 64, keep a
// running row maximum and row sum, and accumulate O.
//
// Shape of the computation on CDNA4: the block's 4 waves own 32 query rows each; two blocks share a
// compute unit (two waves per SIMD) so one wave's softmax overlaps the other's products.  Scores are
// produced transposed, S^T = K Q^T (A = K rows from LDS, B = Q held in registers), so that every
// lane owns one query row: row max / row sum need one cross-lane exchange per tile and the
// accumulator registers of S^T are, as they stand, the B operand of O^T += V^T P^T.  V^T is read
// from the row-major V tile with LDS transpose loads.  K and V tiles are double-buffered in LDS and
// filled by direct global->LDS loads issued one tile ahead; operand fragments are read from LDS a
// few products ahead of their use.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "mfma_utils.h"

namespace slimattn {
namespace {

constexpr int kFwdBQ = 128;   // query rows per block: 4 waves x 32 rows
constexpr int kFwdBK = 64;    // keys per step
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;  // rescale the accumulators only when a row maximum grew by more than 2^8

// One 64-key tile for this wave's 32 query rows.  MASKED tiles touch the diagonal.
// pk[ks]: this lane's K-fragment address for key block 0 and head-dim step ks; pv[db][0..1]: its
// V^T-fragment address pair for head-dim block db; both already point into the current buffer.
// qf holds q * scale * log2(e), so the products are scores in log2 units; the accumulators start
// at minus the row's reference maximum m_ref, so they come out as the exponents directly.
__device__ __forceinline__ int fbits(float x) { return __builtin_bit_cast(int, x); }

template <int D, bool MASKED, class Side>
__device__ __forceinline__ void fwd_tile(const lds_cptr (&pk)[D / 16], const lds_cptr (&pv)[D / 32][2],
                                         const bf16x8 (&qf)[D / 16], floatx16 (&oacc)[D / 32], float& m_ref, float& l_run,
                                         int rel, Side&& side) {
  constexpr int NKS = D / 16, NDB = D / 32, kRowBytes = D * 2;
  floatx16 sacc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[b][r] = -m_ref;
  // S^T = K Q^T (minus the reference maximum)
  // (the next tile's global->LDS loads are issued one at a time between the products)
  frag_pipeline_side<2 * NKS, 4>([&](int i) { return lds_ld_row(pk[i % NKS], (i / NKS) * 32 * kRowBytes); },
                                 [&](int i, bf16x8 f) { sacc[i / NKS] = mfma32(f, qf[i % NKS], sacc[i / NKS]); }, side);
  if (MASKED) {      // key (j0 + 32b + 8(r/4) + 4 half + r%4) > row  <=>  32b + 8(r/4) + r%4 > rel
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * b + 8 * (r >> 2) + (r & 3) > rel) sacc[b][r] = -INFINITY;
  }
  {
    // Lazy rescaling: the reference only moves when some row's tile maximum exceeds it by more than
    // 2^kLazy (wave-uniform test).  Probabilities may therefore exceed 1 by at most that factor;
    // O / l is unaffected.  The reference starts at the row's score against the sample's first key
    // (always visible), so m_ref <= true running maximum (+ rounding) <= m_ref + kLazy throughout
    // and row sums cannot underflow.  Only a positive excess matters, and positive floats
    // order like their bit patterns, so the maximum is taken on the bit patterns as integers
    // (a row whose scores are all below the reference yields some negative value: no rescale).
    int t4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      t4[c] = max(max(fbits(sacc[0][4 * c]), fbits(sacc[0][4 * c + 1])), fbits(sacc[0][4 * c + 2]));
      t4[c] = max(max(t4[c], fbits(sacc[0][4 * c + 3])), fbits(sacc[1][4 * c]));
      t4[c] = max(max(t4[c], fbits(sacc[1][4 * c + 1])), fbits(sacc[1][4 * c + 2]));
      t4[c] = max(t4[c], fbits(sacc[1][4 * c + 3]));
    }
    int imax = max(max(max(t4[0], t4[1]), t4[2]), t4[3]);
    imax = max(imax, __shfl_xor(imax, 32));
    if (__any(imax > fbits(kLazy))) {
      const float shift = imax > 0 ? __builtin_bit_cast(float, imax) : 0.f;
      const float alpha = __builtin_amdgcn_exp2f(-shift);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[b][r] -= shift;
      m_ref += shift;
    }
  }
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[b][r] = __builtin_amdgcn_exp2f(sacc[b][r]);
  bf16x8 pf[4];
  float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks2 = 0; ks2 < 4; ++ks2) {
    pf[ks2] = pack8(sacc[ks2 >> 1], 8 * (ks2 & 1));
    ps[ks2] = sum8(pf[ks2], ps[ks2]);             // row sum of the rounded probabilities the product uses
  }
  l_run += (ps[0] + ps[1]) + (ps[2] + ps[3]);
  // O^T += V^T P^T: one batch of four V^T fragments (the four 16-key steps) per head-dim block
  Tr4 tb[NDB];
  constexpr int kStep = 16 * kRowBytes;
  tr4_issue<0, kStep, 2 * kStep, 3 * kStep>(pv[0][0], pv[0][1], tb[0]);
#pragma unroll
  for (int db = 0; db < NDB; ++db) {
    if (db + 1 < NDB) tr4_issue_wait<0, kStep, 2 * kStep, 3 * kStep>(pv[db + 1][0], pv[db + 1][1], tb[db + 1], tb[db]);
    else tr4_wait(tb[db]);
#pragma unroll
    for (int j = 0; j < 4; ++j) oacc[db] = mfma32(tr4_frag(tb[db], j), pf[j], oacc[db]);
  }
}

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_bf16_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                          const bf16* __restrict__ v, bf16* __restrict__ o,
                                                          float* __restrict__ lse, const QItem* __restrict__ items,
                                                          int n_items, int T, int Hq, int Hkv, float scale) {
  constexpr int NKS = D / 16;   // contraction steps over the head dimension
  constexpr int NDB = D / 32;   // 32-wide blocks of the head dimension
  constexpr int kTileBytes = kFwdBK * D * 2, kBufBytes = 2 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char smem[2 * kBufBytes];   // [buffer][K tile, V tile]

  const int g = Hq / Hkv;
  int item_idx, hk, hg;
  if (!map_block(blockIdx.x, g, Hkv, n_items, &item_idx, &hk, &hg)) return;
  const int h = hk * g + hg;
  const QItem it = items[item_idx];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int q0w = it.q_row0 + 32 * wave;          // first query row of this wave
  const int my_row = q0w + l32;                   // the query row this lane owns
  const int q_end = it.q_row0 + it.q_rows;
  LDS_PTR(char) lds = (LDS_PTR(char))smem;

  const int n_tiles = (q_end - it.kv_start + kFwdBK - 1) / kFwdBK;
  const TileSource srcK = make_tile_source<D, 256>(k, it.kv_start, Hkv, hk, q_end, tid);
  const TileSource srcV = make_tile_source<D, 256>(v, it.kv_start, Hkv, hk, q_end, tid);
  stage_tile<D, kFwdBK, 256>(lds, srcK, 0, tid);
  stage_tile<D, kFwdBK, 256>(lds + kTileBytes, srcV, 0, tid);

  bf16x8 qf[NKS];
  {
    const bf16* qp = q + ((size_t)min(my_row, T - 1) * Hq + h) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = scale8(*reinterpret_cast<const bf16x8*>(qp + 16 * ks), scale * kLog2e);
  }
  lds_cptr pk[NKS], pv[NDB][2];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) pk[ks] = lds_row_ptr<D>(lds, l32, 16 * ks + 8 * half);
#pragma unroll
  for (int db = 0; db < NDB; ++db) lds_tr_ptrs<D>(lds + kTileBytes, 32 * db, lane, pv[db][0], pv[db][1]);
  floatx16 oacc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  // reference maximum (log2 units): the row's score against the first key of the sample
  float m_ref = 0.f, l_run = 0.f;
  {
    const bf16* kp = k + ((size_t)it.kv_start * Hkv + hk) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(kp + 16 * ks);
#pragma unroll
      for (int e = 0; e < 8; ++e) m_ref = fmaf((float)qf[ks][e], (float)k0[e], m_ref);
    }
    m_ref += xor32(m_ref);
  }
  __builtin_amdgcn_s_waitcnt(0);                  // tile 0 has landed in LDS
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = it.kv_start + t * kFwdBK;
    // next tile straight into the other buffer (its last readers passed the barrier below); past
    // the end of the tensor the loads return zeros that nobody uses.  kPasses loads per tensor,
    // spread over the first products of the tile.
    const int nb = ((t + 1) & 1) * kBufBytes;
    constexpr int kPasses = kFwdBK * D * 2 / 256 / 16;
    auto side = [&](int i) {
      if (i < kPasses) stage_pass<D, 256>(lds + nb, srcK, (t + 1) * kFwdBK, i, tid);
      else if (i < 2 * kPasses) stage_pass<D, 256>(lds + nb + kTileBytes, srcV, (t + 1) * kFwdBK, i - kPasses, tid);
    };
    const int rel = my_row - j0 - 4 * half;
    if (j0 + kFwdBK - 1 <= q0w) {                  // whole tile visible to every row of the wave
      fwd_tile<D, false>(pk, pv, qf, oacc, m_ref, l_run, rel, side);
    } else if (j0 <= q0w + 31) {                   // diagonal region
      fwd_tile<D, true>(pk, pv, qf, oacc, m_ref, l_run, rel, side);
    } else {                                       // nothing visible to this wave: only fetch
#pragma unroll
      for (int i = 0; i < 2 * kPasses; ++i) side(i);
    }
    const int flip = (t & 1) ? -kBufBytes : kBufBytes;   // fragment addresses follow the buffer switch
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) pk[ks] += flip;
#pragma unroll
    for (int db = 0; db < NDB; ++db) { pv[db][0] += flip; pv[db][1] += flip; }
    __builtin_amdgcn_s_waitcnt(0);                // this thread's direct loads have landed
    __syncthreads();
  }

  const float l_tot = l_run + xor32(l_run);
  if (my_row < q_end) {
    const float inv = 1.f / l_tot;
    bf16* op = o + ((size_t)my_row * Hq + h) * D;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = (bf16)(oacc[db][4 * gq + x] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq + 4 * half) = w;
      }
    if (half == 0) lse[(size_t)h * T + my_row] = (m_ref + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}


// ---- two-group variant ----------------------------------------------------------------------------
// Used when the query heads per KV head are even.  A block has 8 waves in two groups of 4: both
// groups work on the same 128 query rows and the same K/V tiles (staged once for both) but on two
// different query heads of the KV group.  A wave's tile work is split into a product phase
// M(j) = { S^T(j+1) = K(j+1) Q^T ; O^T += V(j)^T P(j)^T } (matrix cores + LDS reads only) and a
// softmax phase X(j+1) (vector ALU only), and the groups run them in opposite slots: while one
// group's products occupy the matrix cores and the LDS, the other group's softmax runs on the
// vector ALUs of the same SIMDs (at raised wave priority: a wave that streams products would
// otherwise keep the vector issue port to itself).
//
//   slot      0          1      2      3      4
//   group 0   S(0) X(0)  M(0)   X(1)   M(1)   X(2) ...
//   group 1   S(0)       X(0)   M(0)   X(1)   M(1) ...
//
// Two block barriers per tile keep the groups in step.  One closes a group's softmax phase; the
// other sits inside the product phase, two operand batches before its end, after a wait for all of
// the wave's LDS reads: the other group then starts fetching its first operands while this wave's
// last products drain, and every read of the phase is known to be complete at the barrier.
// K(j+2) and V(j+1) are loaded into the buffers of K(j) and V(j-1) by every wave at the start of
// its M(j); those buffers were last read in the other group's M(j-1), behind that barrier.

// Products of one phase for this wave.  All operand fragments come through asm batches of LDS
// reads (row reads for K, transpose reads for V), kDepth batches ahead of their use; KOFF / VOFF
// select the K and V buffers (byte offsets folded into the instructions' immediates).
struct NoHandoff { __device__ __forceinline__ void operator()() const {} };

// `handoff()` runs when only kTail batches are left, all of them already issued: the caller waits
// there for its outstanding LDS reads and passes the block barrier, so that the other group starts
// fetching its first operands while this wave's last products drain.
template <int D, bool DO_S, bool DO_PV, int KOFF, int VOFF, class Handoff = NoHandoff>
__device__ __forceinline__ void fwd_products(const lds_cptr (&pk)[D / 16], const lds_cptr (&pv)[D / 32][2],
                                             const bf16x8 (&qf)[D / 16], floatx16 (&sacc)[2],
                                             const bf16x8 (&pf)[4], floatx16 (&oacc)[D / 32], float m_ref,
                                             Handoff&& handoff = NoHandoff{}) {
  constexpr int NKS = D / 16, NDB = D / 32, kRowBytes = D * 2, kStep = 16 * kRowBytes;
  // A batch of S^T covers one head-dim step for both 32-key blocks (2 reads); a batch of O^T covers
  // one 16-key step for two head-dim blocks (4 reads): consecutive products go to different
  // accumulators, so a wave that has the matrix core to itself does not wait on its own previous
  // product.
  constexpr int NSU = DO_S ? NKS : 0, NPU = DO_PV ? 2 * NDB : 0, NU = NSU + NPU;
  constexpr int kDepth = 3, kTail = 2, kKb = 32 * kRowBytes;
  static_assert(kTail < kDepth, "the tail batches must have been issued before the handoff");
  R2 ru[NSU ? NSU : 1];
  Tr2 tu[NPU ? NPU : 1];
  if (DO_S) {   // 64-bit moves: half as many instructions on the vector port as 32-bit ones
    typedef __attribute__((__vector_size__(8 * sizeof(double)))) double doublex8;
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
    const floatx2 mm = {-m_ref, -m_ref};
    const double m2 = __builtin_bit_cast(double, mm);
    const doublex8 init = {m2, m2, m2, m2, m2, m2, m2, m2};
    sacc[0] = __builtin_bit_cast(floatx16, init);
    sacc[1] = __builtin_bit_cast(floatx16, init);
  }
  auto issue = [&](auto ic) {
    constexpr int u = decltype(ic)::value;
    if constexpr (u < NSU) {
      r2_issue<KOFF, KOFF + kKb>(pk[u], pk[u], ru[u]);
    } else {
      constexpr int x = u - NSU, ks = x / (NDB / 2), dp = x % (NDB / 2);
      tr2x_issue<VOFF + ks * kStep>(pv[2 * dp][0], pv[2 * dp][1], pv[2 * dp + 1][0], pv[2 * dp + 1][1], tu[x]);
    }
  };
  auto consume = [&](auto ic) {
    constexpr int u = decltype(ic)::value;
    // LDS reads issued after batch u by the time it is consumed: batches u+1 .. u+kDepth
    constexpr int last = (u + kDepth < NU - 1) ? u + kDepth : NU - 1;
    constexpr int n_s = (last < NSU ? last + 1 : NSU) - (u + 1 < NSU ? u + 1 : NSU);
    constexpr int behind = 2 * n_s + 4 * ((last - u) - n_s);
    if constexpr (u < NSU) {
      lds_wait<behind>(ru[u]);
#pragma unroll
      for (int j = 0; j < 2; ++j) sacc[j] = mfma32(ru[u].f[j], qf[u], sacc[j]);
    } else {
      constexpr int x = u - NSU, ks = x / (NDB / 2), dp = x % (NDB / 2);
      lds_wait<behind>(tu[x]);
#pragma unroll
      for (int j = 0; j < 2; ++j) oacc[2 * dp + j] = mfma32(tr2_frag(tu[x], j), pf[ks], oacc[2 * dp + j]);
    }
  };
  static_for<0, (NU < kDepth ? NU : kDepth)>(issue);
  static_for<0, NU>([&](auto ic) {
    constexpr int u = decltype(ic)::value;
    if constexpr (u + kDepth < NU) issue(IC<u + kDepth>{});
    consume(ic);
    __builtin_amdgcn_sched_barrier(0);             // keep the products next to their batch
    if constexpr (u == NU - 1 - kTail) {
      handoff();
      __builtin_amdgcn_sched_barrier(0);
    }
  });
}

// Softmax phase: exponents in sacc (scores in log2 units minus m_ref) -> packed probabilities pf,
// row sum, lazy rescale of the accumulators (see fwd_tile for the argument).
template <int D>
__device__ __forceinline__ void fwd_softmax(floatx16 (&sacc)[2], bf16x8 (&pf)[4], floatx16 (&oacc)[D / 32], float& m_ref,
                                            float& l_run, int rel, bool masked) {
  constexpr int NDB = D / 32;
  if (masked) {    // wave-uniform: the tile touches or lies beyond the diagonal of some row of the wave
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (32 * b + 8 * (r >> 2) + (r & 3) > rel) sacc[b][r] = -INFINITY;
  }
  int t4[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    t4[c] = max(max(fbits(sacc[0][4 * c]), fbits(sacc[0][4 * c + 1])), fbits(sacc[0][4 * c + 2]));
    t4[c] = max(max(t4[c], fbits(sacc[0][4 * c + 3])), fbits(sacc[1][4 * c]));
    t4[c] = max(max(t4[c], fbits(sacc[1][4 * c + 1])), fbits(sacc[1][4 * c + 2]));
    t4[c] = max(t4[c], fbits(sacc[1][4 * c + 3]));
  }
  int imax = max(max(max(t4[0], t4[1]), t4[2]), t4[3]);
  {   // maximum over the two half-waves that share a query row (lane l and lane l ^ 32)
    const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)imax, (unsigned)imax, false, false);
    imax = max((int)sw[0], (int)sw[1]);
  }
  if (__any(imax > fbits(kLazy))) {
    const float shift = imax > 0 ? __builtin_bit_cast(float, imax) : 0.f;
    const float alpha = __builtin_amdgcn_exp2f(-shift);
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[b][r] -= shift;
    m_ref += shift;
  }
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[b][r] = __builtin_amdgcn_exp2f(sacc[b][r]);
  float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks2 = 0; ks2 < 4; ++ks2) {
    pf[ks2] = pack8(sacc[ks2 >> 1], 8 * (ks2 & 1));
    ps[ks2] = sum8(pf[ks2], ps[ks2]);
  }
  l_run += (ps[0] + ps[1]) + (ps[2] + ps[3]);
}

template <int D>
__global__ __launch_bounds__(512, 2) void fwd_pair_bf16_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                               const bf16* __restrict__ v, bf16* __restrict__ o,
                                                               float* __restrict__ lse, const QItem* __restrict__ items,
                                                               int n_items, int T, int Hq, int Hkv, float scale) {
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int kTileBytes = kFwdBK * D * 2, kBufBytes = 2 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char smem[2 * kBufBytes];   // [buffer][K tile, V tile]

  const int g = Hq / Hkv;
  int item_idx, hk, hp;
  if (!map_block(blockIdx.x, g >> 1, Hkv, n_items, &item_idx, &hk, &hp)) return;
  const QItem it = items[item_idx];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int grp = __builtin_amdgcn_readfirstlane(wave >> 2), w4 = __builtin_amdgcn_readfirstlane(wave & 3);
  const int h = hk * g + 2 * hp + grp;
  const int q0w = it.q_row0 + 32 * w4;
  const int my_row = q0w + l32;
  const int q_end = it.q_row0 + it.q_rows;
  LDS_PTR(char) lds = (LDS_PTR(char))smem;

  const int n_tiles = (q_end - it.kv_start + kFwdBK - 1) / kFwdBK;
  // tiles this wave sees without a mask (a prefix of the tile sequence)
  const int n_full = max(0, (q0w - it.kv_start + 1) / kFwdBK);
  // The block's global loads are all issued before anything waits: the Q rows first, then the first
  // tiles.  One memory latency is then paid once per block.
  bf16x8 qf[NKS];
  {
    const bf16* qp = q + ((size_t)min(my_row, T - 1) * Hq + h) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
  }
  const TileSource srcK = make_tile_source<D, 512>(k, it.kv_start, Hkv, hk, q_end, tid);
  const TileSource srcV = make_tile_source<D, 512>(v, it.kv_start, Hkv, hk, q_end, tid);
  stage_tile<D, kFwdBK, 512>(lds, srcK, 0, tid);
  stage_tile<D, kFwdBK, 512>(lds + kTileBytes, srcV, 0, tid);
  stage_tile<D, kFwdBK, 512>(lds + kBufBytes, srcK, kFwdBK, tid);

  lds_cptr pk[NKS], pv[NDB][2];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) pk[ks] = lds_row_ptr<D>(lds, l32, 16 * ks + 8 * half);
#pragma unroll
  for (int db = 0; db < NDB; ++db) lds_tr_ptrs<D>(lds + kTileBytes, 32 * db, lane, pv[db][0], pv[db][1]);
  floatx16 oacc[NDB], sacc[2];
  bf16x8 pf[4];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m_ref = 0.f, l_run = 0.f;
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) qf[ks] = scale8(qf[ks], scale * kLog2e);

  const int rel0 = my_row - it.kv_start - 4 * half;      // rel of tile t = rel0 - t * kFwdBK
  // A tile beyond the wave's last visible one is treated as fully masked (its probabilities are
  // zero), so every wave runs the same straight-line loop body; the waves concerned would
  // otherwise wait at the barriers for the block's lower rows.
  // slot 0: S(0) for both groups, X(0) for group 0 only
  fwd_products<D, true, false, 0, 0>(pk, pv, qf, sacc, pf, oacc, m_ref);
  {
    // Reference maximum (log2 units): the row's score against the first key of the sample, which
    // every row sees.  It is element [key 0][row] of S^T(0): register 0 of the lower half-wave.
    m_ref = __shfl(sacc[0][0], l32);                // both halves take the lower half's value
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[b][r] -= m_ref;
  }
  if (grp) __syncthreads();
  fwd_softmax<D>(sacc, pf, oacc, m_ref, l_run, rel0, n_full < 1);
  __syncthreads();

  // One loop iteration: M(j) then X(j+1).  K(j+1) sits in buffer (j+1) & 1 and V(j) in buffer j & 1;
  // the loop is unrolled by that parity so that every LDS offset is an immediate.
  auto handoff = [&]() {
    // group 1's loads must have landed before group 0 starts M(j+1) behind this barrier; group 0's
    // own loads are waited for at the end of its softmax phase
    if (grp) __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0xc07f);       // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };
#define SLIMATTN_FWD_ITER(PAR)                                                                                     \
  {                                                                                                                \
    /* loads for K(j+2), V(j+1) (past the tensor's end they return zeros nobody uses): their buffers were last */  \
    /* read in the other group's M(j-1), whose reads completed before the barrier this wave has just passed */     \
    stage_tile<D, kFwdBK, 512>(lds + (PAR) * kBufBytes, srcK, (j + 2) * kFwdBK, tid);                              \
    stage_tile<D, kFwdBK, 512>(lds + (1 - (PAR)) * kBufBytes + kTileBytes, srcV, (j + 1) * kFwdBK, tid);           \
    fwd_products<D, true, true, (1 - (PAR)) * kBufBytes, (PAR) * kBufBytes>(pk, pv, qf, sacc, pf, oacc, m_ref, handoff); \
    /* a wave streaming products would otherwise keep the vector issue port to itself */                        \
    __builtin_amdgcn_s_setprio(3);                                                                                 \
    fwd_softmax<D>(sacc, pf, oacc, m_ref, l_run, rel0 - (j + 1) * kFwdBK, j + 1 >= n_full);                        \
    __builtin_amdgcn_s_setprio(0);                                                                                 \
    __builtin_amdgcn_s_waitcnt(0x0f70); /* vmcnt(0) */                                                             \
    __builtin_amdgcn_s_barrier();                                                                                  \
  }
  int j = 0;
  for (; j + 2 < n_tiles; j += 2) {
    SLIMATTN_FWD_ITER(0)
    ++j;
    SLIMATTN_FWD_ITER(1)
    --j;
  }
  if (j + 1 < n_tiles) {
    SLIMATTN_FWD_ITER(0)
    ++j;
  }
#undef SLIMATTN_FWD_ITER
  // M(n_tiles - 1): the last O^T update; V(j) sits in buffer j & 1
  if (j & 1) fwd_products<D, false, true, 0, kBufBytes>(pk, pv, qf, sacc, pf, oacc, m_ref);
  else fwd_products<D, false, true, 0, 0>(pk, pv, qf, sacc, pf, oacc, m_ref);

  const float l_tot = l_run + xor32(l_run);
  if (my_row < q_end) {
    const float inv = 1.f / l_tot;
    bf16* op = o + ((size_t)my_row * Hq + h) * D;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = (bf16)(oacc[db][4 * gq + x] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * db + 8 * gq + 4 * half) = w;
      }
    if (half == 0) lse[(size_t)h * T + my_row] = (m_ref + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
  if (!grp) __syncthreads();                       // group 1 passed one more barrier in slot 0
}

}  // namespace

int fwd_q_tile(int dtype, int) { return dtype == SLIMATTN_F32 ? 64 : kFwdBQ; }

int launch_fwd_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, void* o, float* lse,
                    const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const int g = p.n_q_heads / p.n_kv_heads;
  if (g % 2 == 0 && p.head_dim == 128) return launch_fwd_wide_bf16(c, q, k, v, o, lse, items, n_items);
  if (g % 2 == 0) {
    const dim3 grid(mapped_grid(n_items, p.n_kv_heads, g / 2)), block(512);
    if (p.head_dim == 128)
      hipLaunchKernelGGL(fwd_pair_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                         (const bf16*)v, (bf16*)o, lse, items, n_items, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale);
    else
      hipLaunchKernelGGL(fwd_pair_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                         (const bf16*)v, (bf16*)o, lse, items, n_items, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale);
    return (int)hipGetLastError();
  }
  const dim3 grid(mapped_grid(n_items, p.n_kv_heads, g)), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(fwd_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (bf16*)o, lse, items, n_items, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale);
  else
    hipLaunchKernelGGL(fwd_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (bf16*)o, lse, items, n_items, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale);
  return (int)hipGetLastError();
}

}  // namespace slimattn
