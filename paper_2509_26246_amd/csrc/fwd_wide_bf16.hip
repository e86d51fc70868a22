// Forward for bf16 inputs and an even number of query heads per KV head: one wave per SIMD.
//
// What it computes is the forward of fwd_bf16.hip (a query tile of 128 rows attends to the sample's keys
// kv_start .. its last row, online softmax in log2 units, O and lse out); a block is 4 waves, each wave
// owns 32 query rows of TWO query heads of one KV group, and the block walks the K/V tiles (64 keys) once
// for both heads.
//
// Shape on CDNA4.  With one wave per SIMD the O^T accumulators of both heads (128 registers at head dim
// 128) live in the accumulation half of the register file, touched only by products issued from inline asm,
// and every K and V^T fragment read from LDS feeds two products (one per head): 0.75 LDS reads per
// product.  Nothing else runs on the SIMD, so the wave overlaps its own work: behind each product (32
// cycles of the matrix unit, 4 to issue) there is room for one LDS read and the element-wise work of one
// score, and the code is written slot by slot so that exactly this is there.  The unit of the software
// pipeline is half a tile (32 keys, "unit" below): while the scores of unit h+1 are produced (16 products)
// and the O^T update of unit h-1 runs (16 products), the 32 scores per lane of unit h are turned into
// packed probabilities, one per slot:
//   iteration t:  [S(t+1, kb 0) | EW(t, kb 1) first half]   [PV(t, kb 0) | EW(t, kb 1) second half]
//                 [S(t+1, kb 1) | EW(t+1, kb 0) first half] [PV(t, kb 1) | EW(t+1, kb 0) second half]  barrier
// K(t+2) and V(t+1) are staged global -> LDS during iteration t into the buffers iteration t-1 read (the first
// iteration, which has no tile before it, stages nothing: K(0), K(1), V(0) come with the item's first loads).
//
// Softmax reference.  A row's reference m is its score against the sample's first key (every row sees it),
// computed in the prologue; the first product of a score accumulator takes -m as its C operand from a
// register block that holds it (no initialisation, no vector instructions), so the products deliver the
// exponents.  The
// exponentials of a unit are taken against the reference as it stands; when the unit is done and before
// its probabilities are used, one wave-uniform test asks whether any lane's sum of the unit's 16 probabilities
// of a head exceeded 2^12 (an overflow to inf trips it too), and only then the reference moves: accumulators and
// row sums are rescaled, the unit's probabilities recomputed from its scores (still in their registers) and the
// next unit's scores shifted.
//
// Hazards of the inline-asm products: see dkdv_wide_bf16.hip; here their results (O^T) are read only by
// later products on the same accumulator, and after explicit wait states in the rescaling path and the
// epilogue; their B operands (packed probabilities) were written at least one phase earlier.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "mfma_utils.h"

namespace slimattn {
namespace {

constexpr int kKeys = 64;                               // keys per tile: two units of 32
template <int D> constexpr int kNKS = D / 16;           // head-dim steps of a score product
template <int D> constexpr int kNDB = D / 32;           // head-dim blocks of an O^T accumulator
template <int D> constexpr int kNVF = 2 * kNDB<D>;      // V^T fragments of a unit: 2 key steps x head-dim blocks
template <int D> constexpr int kRowBytes = D * 2;
template <int D> constexpr int kTileBytes = kKeys * kRowBytes<D>;
template <int D> constexpr int kVBase = 2 * kTileBytes<D>;   // LDS: K buffer 0, K buffer 1, V buffer 0, V buffer 1
template <int D> constexpr int kPer = 128 / D;          // element-wise values per product slot
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// the reference moves when a lane's sum of the 16 probabilities of a unit and head exceeds this (so no
// single one does; an overflow to inf does)
constexpr float kLazySum = 4096.f;

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned uintx4;
__device__ __forceinline__ bf16x8 as_frag(uintx4 x) { return __builtin_bit_cast(bf16x8, x); }
__device__ __forceinline__ int fbits(float x) { return __builtin_bit_cast(int, x); }

struct Tr1 { short4v r[2]; };                           // one transposed fragment: two 64-bit reads
__device__ __forceinline__ bf16x8 tr1_frag(const Tr1& t) {
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short short8v;
  short8v x = __builtin_shufflevector(t.r[0], t.r[1], 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, x);
}
template <int N>
__device__ __forceinline__ void wait_k(bf16x8& f) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f) : "n"(N)); }
template <int N>
__device__ __forceinline__ void wait_v(Tr1& t) { asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(t.r[0]), "+v"(t.r[1]) : "n"(N)); }

__device__ __forceinline__ void mfma_acc(floatx16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// acc += a b with the accumulator in architectural registers.  An asm statement like the others of a slot, so
// that the order "product, then what hides behind it" is the written one (a builtin product was moved behind
// its slot's other instructions, two products then met back to back and the second one's wait for the
// matrix unit kept the vector instructions behind it from issuing).
__device__ __forceinline__ void mfma_v(floatx16& acc, bf16x8 a, bf16x8 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// acc = a b + c: the first product of a score accumulator takes minus the reference from a register block of
// its own (every register of c holds -m of the lane's row), so the accumulators need no initialisation.
__device__ __forceinline__ void mfma_v_from(floatx16& acc, bf16x8 a, bf16x8 b, const floatx16& c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(acc) : "v"(a), "v"(b), "v"(c));
}
__device__ __forceinline__ void settle_writes(floatx16& a, floatx16& b) { asm volatile("s_nop 7" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void settle2(floatx16& a, floatx16& b) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void lds_ptr_add(lds_cptr& p, int d) {
  unsigned x = (unsigned)(size_t)p;
  asm volatile("v_add_u32 %0, %1, %0" : "+v"(x) : "s"(d));
  p = (lds_cptr)(size_t)x;
}

// Element-wise work of one unit (kb = KE) as a stream of 32 values, value J = register J % 16 of head
// J / 16, one slot per value; each slot is one asm statement (stays where it is written, no wait states
// added).  Slot J: the exponential of value J, the row-sum update with value J - 1 (in fp32, before the
// rounding to bf16), and in even slots the packing of the pair (J-2, J-1).  Slots 0 and 1 also add the
// previous unit's row sums to the running ones.  No instruction reads the result of the
// exponential right in front of it (a transcendental's result is not forwarded to the next instruction).
// (Row sums over the packed values with the dot-product instruction, as the two-wave kernel takes them,
// are not used here: that instruction did not overlap with a running matrix product.)
template <int KE, int J>
__device__ __forceinline__ void ew_slot(floatx16 (&s)[2][2], uintx4 (&pf)[2][2][2], float& e0, float& e1, float (&lr)[2],
                                        float (&lu)[2]) {
  constexpr int hb = J >> 4, r = J & 15;
  const float x = s[hb][KE][r];
  if constexpr (J == 0) {
    asm volatile("v_exp_f32 %0, %3\n\tv_add_f32 %1, %1, %2" : "=&v"(e0), "+v"(lr[0]) : "v"(lu[0]), "v"(x));
  } else if constexpr (J == 1) {
    asm volatile("v_exp_f32 %0, %4\n\tv_add_f32 %1, %1, %3\n\tv_mov_b32 %2, %5"
                 : "=&v"(e1), "+v"(lr[1]), "=&v"(lu[0])
                 : "v"(lu[1]), "v"(x), "v"(e0));
  } else if constexpr (J == 17) {
    asm volatile("v_exp_f32 %0, %2\n\tv_mov_b32 %1, %3" : "=&v"(e1), "=&v"(lu[1]) : "v"(x), "v"(e0));
  } else if constexpr (J & 1) {
    asm volatile("v_exp_f32 %0, %2\n\tv_add_f32 %1, %1, %3" : "=&v"(e1), "+v"(lu[hb]) : "v"(x), "v"(e0));
  } else {
    constexpr int pe = J - 1, phb = pe >> 4, pr = pe & 15;     // pack the pair (J - 2, J - 1)
    unsigned w;
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %3\n\tv_exp_f32 %1, %4\n\tv_add_f32 %2, %2, %3"
                 : "=&v"(w), "+v"(e0), "+v"(lu[phb])
                 : "v"(e1), "v"(x));
    pf[phb][KE][pr >> 3][(pr & 7) >> 1] = w;
  }
}
// behind slot 31: the last pair and its row-sum update
template <int KE>
__device__ __forceinline__ void ew_flush(uintx4 (&pf)[2][2][2], float& e0, float& e1, float (&lu)[2]) {
  unsigned w;
  asm volatile("v_cvt_pk_bf16_f32 %0, %2, %3\n\tv_add_f32 %1, %1, %3" : "=&v"(w), "+v"(lu[1]) : "v"(e0), "v"(e1));
  pf[1][KE][1][3] = w;
}

template <int D>
__device__ __forceinline__ void fwd_wide_item(const QItem it, const int hk, const int hp, const bf16* __restrict__ q,
                                              const bf16* __restrict__ k, const bf16* __restrict__ v, bf16* __restrict__ o_out,
                                              float* __restrict__ lse, int T, int Hq, int Hkv, float scale) {
  constexpr int NKS = kNKS<D>, NDB = kNDB<D>, NVF = kNVF<D>, PER = kPer<D>;
  // K and V buffers, then one transposition area per wave for the output rows (row stride padded by 16 bytes)
  constexpr int kOutStride = kRowBytes<D> + 16, kOutBytes = 32 * kOutStride;
  __shared__ __attribute__((aligned(1024))) char smem[4 * kTileBytes<D> + 4 * kOutBytes];

  const int g = Hq / Hkv;
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int h0 = hk * g + 2 * hp;
  const int q0w = it.q_row0 + 32 * wave, my_row = q0w + l32, q_end = it.q_row0 + it.q_rows;
  LDS_PTR(char) lds = (LDS_PTR(char))smem;
  const int n_tiles = (q_end - it.kv_start + kKeys - 1) / kKeys;
  // tiles this wave sees without a mask (at most all: a wave past the end of a ragged query tile)
  const int n_full = min(max(0, (q0w - it.kv_start + 1) / kKeys), n_tiles);

  // all of the block's first loads are issued before anything waits
  bf16x8 qf[2][NKS], k0[NKS];
#pragma unroll
  for (int hb = 0; hb < 2; ++hb) {
    const bf16* qp = q + ((size_t)min(my_row, T - 1) * Hq + h0 + hb) * D + 8 * half;
#pragma unroll
    for (int u = 0; u < NKS; ++u) qf[hb][u] = *reinterpret_cast<const bf16x8*>(qp + 16 * u);
  }
  {
    const bf16* kp = k + ((size_t)it.kv_start * Hkv + hk) * D + 8 * half;
#pragma unroll
    for (int u = 0; u < NKS; ++u) k0[u] = *reinterpret_cast<const bf16x8*>(kp + 16 * u);
  }
  const TileSource srcK = make_tile_source<D, 256>(k, it.kv_start, Hkv, hk, q_end, tid);
  const TileSource srcV = make_tile_source<D, 256>(v, it.kv_start, Hkv, hk, q_end, tid);
  // K(0), K(1) and V(0) are on their way before anything waits: one memory latency per item, not one per early tile
  stage_tile<D, kKeys, 256>(lds, srcK, 0, tid);
  stage_tile<D, kKeys, 256>(lds + kTileBytes<D>, srcK, kKeys, tid);
  stage_tile<D, kKeys, 256>(lds + kVBase<D>, srcV, 0, tid);

  lds_cptr pk[NKS], pv[NDB][2];                         // fragment addresses: K buffer 0, V buffer 0
#pragma unroll
  for (int u = 0; u < NKS; ++u) pk[u] = lds_row_ptr<D>(lds, l32, 16 * u + 8 * half);
#pragma unroll
  for (int db = 0; db < NDB; ++db) lds_tr_ptrs<D>(lds + kVBase<D>, 32 * db, lane, pv[db][0], pv[db][1]);

  floatx16 o[2][NDB];                                   // O^T of the two heads: accumulation registers
#pragma unroll
  for (int hb = 0; hb < 2; ++hb)
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
#pragma unroll
      for (int r = 0; r < 16; ++r) o[hb][db][r] = 0.f;
      asm volatile("" : "+a"(o[hb][db]));
    }

  // q * scale * log2 e (rounded to bf16): the products give scores in log2 units; the reference of a row is
  // its score against the sample's first key
  float m_ref[2];
  floatx16 negm[2];                                     // -m in every register: the C operand of an accumulator's first product
#pragma unroll
  for (int hb = 0; hb < 2; ++hb) {
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < NKS; ++u) {
      qf[hb][u] = scale8(qf[hb][u], scale * kLog2e);
#pragma unroll
      for (int x = 0; x < 4; ++x) {                     // packed bf16 pairs, fp32 sum (no product runs yet: see ew_slot)
        const bf16x2 a2 = {qf[hb][u][2 * x], qf[hb][u][2 * x + 1]}, b2 = {k0[u][2 * x], k0[u][2 * x + 1]};
        acc = __builtin_amdgcn_fdot2_f32_bf16(a2, b2, acc, false);
      }
    }
    m_ref[hb] = acc + xor32(acc);
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[hb][r] = -m_ref[hb];
    asm volatile("" : "+v"(negm[hb]));                  // kept in registers, not rebuilt at every use
  }

  floatx16 s[2][2];                                     // S^T [head][key block of the tile]
  uintx4 pf[2][2][2];                                   // packed P^T [head][key block][16-key step]
  float e0 = 0.f, e1 = 0.f, lr[2] = {0.f, 0.f}, lu[2] = {0.f, 0.f};
  int rel_n = my_row - it.kv_start - 4 * half;          // of the tile whose scores come next
  int t = -1;
  int ksoff = kKeys * srcK.row_bytes;                   // byte offset of tile t + 2 in the sample's rows
  const int wave_off = wave * 1024;

  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  // ---- pieces of an iteration -------------------------------------------------------------------
  // Masked tiles: the score accumulators of key block KB are set to -m, or to -inf for pairs past the diagonal
  // (whatever is added later), and every product adds to them.
  auto mask = [&](auto kbc) {
    constexpr int KB = decltype(kbc)::value;
    const int rel = rel_n - 32 * KB;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[hb][KB][r] = (8 * (r >> 2) + (r & 3) > rel) ? -INFINITY : negm[hb][r];
  };
  auto settle = [&]() {                                 // results of the asm products become readable
    if constexpr (NDB == 4)
      asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15"
                   : "+a"(o[0][0]), "+a"(o[0][1]), "+a"(o[0][2]), "+a"(o[0][3]), "+a"(o[1][0]), "+a"(o[1][1]), "+a"(o[1][2]),
                     "+a"(o[1][3]));
    else
      asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+a"(o[0][0]), "+a"(o[0][1]), "+a"(o[1][0]), "+a"(o[1][1]));
  };
  // The reference moves (rare): unit KB has just been turned into probabilities against the old reference
  // and nobody has used them; unit 1 - KB has its scores and waits for its element-wise pass.
  auto move_reference = [&](auto kbc) {
    constexpr int KB = decltype(kbc)::value;
    settle();
    settle2(s[0][1 - KB], s[1][1 - KB]);
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      float mxs = s[hb][KB][0];                         // the unit's largest exponent of the row, both half-waves
#pragma unroll
      for (int r = 1; r < 16; ++r) mxs = fmaxf(mxs, s[hb][KB][r]);
      mxs = fmaxf(mxs, xor32(mxs));
      const float shift = fmaxf(mxs, 0.f);
      const float alpha = __builtin_amdgcn_exp2f(-shift);
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[hb][db][r] *= alpha;
      lr[hb] *= alpha;
      floatx16 e;
#pragma unroll
      for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(s[hb][KB][r] - shift);
      const bf16x8 p0 = pack8(e, 0), p1 = pack8(e, 8);
      pf[hb][KB][0] = __builtin_bit_cast(uintx4, p0);
      pf[hb][KB][1] = __builtin_bit_cast(uintx4, p1);
      float sum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += e[r];
      lu[hb] = sum;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[hb][1 - KB][r] -= shift;
      m_ref[hb] += shift;
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[hb][r] = -m_ref[hb];
      asm volatile("" : "+v"(negm[hb]));
    }
    settle_writes(negm[0], negm[1]);                    // vector writes, then asm products reading them as C operands
  };
  // Start of a score phase: the lazy test for the unit just finished, the mask.
  auto boundary = [&](auto kbc, auto checkc, auto maskc) {
    constexpr int KB = decltype(kbc)::value;
    if constexpr (decltype(checkc)::value != 0) {
      if (__builtin_expect(__any(fmaxf(lu[0], lu[1]) > kLazySum), 0)) move_reference(kbc);
    }
    if constexpr (decltype(maskc)::value != 0) {
      mask(kbc);
      settle_writes(s[0][KB], s[1][KB]);               // vector writes, then asm products reading them
    }
  };

  // MASKED: the tile whose scores are produced touches or lies past the diagonal of some row of the wave.
  auto iteration = [&](auto first_c, auto masked_c) {
    constexpr bool first = decltype(first_c)::value != 0;
    using MaskT = decltype(masked_c);
    const int dbuf = (t & 1) ? kTileBytes<D> : -kTileBytes<D>;   // both pointer sets move to buffer t & 1
    const int kdst = (t & 1) * kTileBytes<D> + wave_off;                       // K(t+2) -> K buffer t & 1
    const int vdst = kVBase<D> + ((t + 1) & 1) * kTileBytes<D> + wave_off;     // V(t+1) -> V buffer (t+1) & 1
    bf16x8 ka[2][NKS];
    Tr1 va[2][NVF];
    constexpr int kPasses = kTileBytes<D> / 4096, kRowsPerPass = 4096 / kRowBytes<D>;
    // Tiles behind the item's last are not fetched: their loads get an offset beyond the tensor (the hardware's range
    // check answers with zeros at once), so that the wait that ends the item's last iterations does not sit out
    // the latency of loads nobody needs; the number of loads per iteration stays fixed.
    constexpr int kBeyond = 0x7FF00000;
    const int ksoff_k = t + 2 < n_tiles ? ksoff : kBeyond;
    const int ksoff_v = t + 1 < n_tiles ? ksoff - kKeys * srcK.row_bytes : kBeyond;

    auto ew = [&](auto kec, auto jc) {                  // the element-wise slots behind product slot j of a half
      constexpr int KE = decltype(kec)::value, j = decltype(jc)::value;
      static_for<0, PER>([&](auto ec) { ew_slot<KE, PER * j + decltype(ec)::value>(s, pf, e0, e1, lr, lu); });
    };
    // Score products of unit (t+1, KB).  NEXT: what the last two fragments' slots prefetch: 1 the unit's first
    // V^T fragments (its O^T update comes next), 2 the K fragments of key block 1, 0 nothing.  EW: the
    // first half of the element-wise work of key block 1 - KB runs in the slots.
    auto phase_s = [&](auto kbc, auto nextc, auto ewc, auto&& extra) {
      constexpr int KB = decltype(kbc)::value, NEXT = decltype(nextc)::value;
      constexpr bool EW = decltype(ewc)::value != 0, kMasked = MaskT::value != 0;
      static_for<0, 2 * NKS>([&](auto pc) {
        constexpr int p = decltype(pc)::value, u = p / 2, hb = p % 2;
        if constexpr (hb == 0) {
          constexpr int N = (u + 1 < NKS) ? 1 : (NEXT == 1 ? 2 : NEXT == 2 ? 1 : 0);
          wait_k<N>(ka[KB][u]);
        }
        if constexpr (u == 0 && !kMasked) mfma_v_from(s[hb][KB], ka[KB][u], qf[hb][u], negm[hb]);
        else mfma_v(s[hb][KB], ka[KB][u], qf[hb][u]);
        if constexpr (u + 2 < NKS) {
          if constexpr (hb == 0) r1_issue<KB * 32 * kRowBytes<D>>(pk[u + 2], ka[KB][u + 2]);
        } else if constexpr (NEXT == 1) {
          constexpr int f = u + 2 - NKS;                // ks = 0, db = f
          tr1_issue<2 * KB * 16 * kRowBytes<D>>(pv[f][hb], va[KB][f].r[hb]);
        } else if constexpr (NEXT == 2) {
          if constexpr (hb == 0) r1_issue<32 * kRowBytes<D>>(pk[u + 2 - NKS], ka[1][u + 2 - NKS]);
        }
        if constexpr (EW) ew(IC<1 - KB>{}, pc);
        extra(pc);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    // O^T update of unit (t, KB).  NEXT: 2 the last two fragments' slots prefetch the K fragments of key
    // block 1, 0 nothing.  The second half of the element-wise work of key block 1 - KB runs in the slots.
    auto phase_pv = [&](auto kbc, auto nextc, auto&& extra) {
      constexpr int KB = decltype(kbc)::value, NEXT = decltype(nextc)::value;
      static_for<0, 2 * NVF>([&](auto pc) {
        constexpr int p = decltype(pc)::value, f = p / 2, hb = p % 2, ks = f / NDB, db = f % NDB;
        if constexpr (hb == 0) {
          constexpr int N = (f + 1 < NVF) ? 2 : (NEXT == 2 ? 1 : 0);
          wait_v<N>(va[KB][f]);
        }
        mfma_acc(o[hb][db], tr1_frag(va[KB][f]), as_frag(pf[hb][KB][ks]));
        if constexpr (f + 2 < NVF) {
          constexpr int f2 = f + 2, ks2 = f2 / NDB, db2 = f2 % NDB;
          tr1_issue<(2 * KB + ks2) * 16 * kRowBytes<D>>(pv[db2][hb], va[KB][f2].r[hb]);
        } else if constexpr (NEXT == 2) {
          if constexpr (hb == 0) r1_issue<32 * kRowBytes<D>>(pk[f + 2 - NVF], ka[1][f + 2 - NVF]);
        }
        ew(IC<1 - KB>{}, IC<2 * NVF + p>{});
        extra(pc);
        __builtin_amdgcn_sched_barrier(0);
      });
      ew_flush<1 - KB>(pf, e0, e1, lu);
    };
    // bookkeeping pieces, one behind a product
    auto extra_a0 = [&](auto pc) {                      // V pointers to this iteration's buffer; K(t+2) staged
      constexpr int p = decltype(pc)::value;
      if constexpr (p < 2 * NDB) lds_ptr_add(pv[p / 2][p % 2], dbuf);
      if constexpr (!first && p > 2 * NDB && (p - 2 * NDB) % 2 == 1 && (p - 2 * NDB) / 2 < kPasses) {
        constexpr int pass = (p - 2 * NDB) / 2;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(srcK.rsrc, lds + kdst + pass * 4096, 16, srcK.voff,
                                                 ksoff_k + pass * kRowsPerPass * srcK.row_bytes, 0, 0);
      }
    };
    auto extra_a1 = [&](auto pc) {                      // V(t+1) staged
      constexpr int p = decltype(pc)::value;
      if constexpr (!first && p > 2 * NDB && (p - 2 * NDB) % 2 == 1 && (p - 2 * NDB) / 2 < kPasses) {
        constexpr int pass = (p - 2 * NDB) / 2;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(srcV.rsrc, lds + vdst + pass * 4096, 16, srcV.voff,
                                                 ksoff_v + pass * kRowsPerPass * srcK.row_bytes, 0, 0);
      }
    };
    auto extra_b1 = [&](auto pc) {                      // K pointers to the next iteration's buffer
      constexpr int p = decltype(pc)::value;
      if constexpr (p < NKS) lds_ptr_add(pk[p], dbuf);
    };
    auto none = [&](auto) {};

    r1_issue<0>(pk[0], ka[0][0]);
    r1_issue<0>(pk[1], ka[0][1]);
    if constexpr (first) {
      boundary(IC<0>{}, IC<0>{}, MaskT{});
      phase_s(IC<0>{}, IC<2>{}, IC<0>{}, extra_a0);
      boundary(IC<1>{}, IC<0>{}, MaskT{});
      phase_s(IC<1>{}, IC<0>{}, IC<1>{}, extra_a1);
      static_for<0, 2 * NVF>([&](auto pc) {             // no O^T update yet: the second half of unit (0, 0) on its own
        ew(IC<0>{}, IC<2 * NVF + decltype(pc)::value>{});
        extra_b1(pc);
      });
      ew_flush<0>(pf, e0, e1, lu);
    } else {
      boundary(IC<0>{}, IC<1>{}, MaskT{});
      phase_s(IC<0>{}, IC<1>{}, IC<1>{}, extra_a0);
      phase_pv(IC<0>{}, IC<2>{}, none);
      boundary(IC<1>{}, IC<1>{}, MaskT{});
      phase_s(IC<1>{}, IC<1>{}, IC<1>{}, extra_a1);
      phase_pv(IC<1>{}, IC<0>{}, extra_b1);
    }
    ksoff += kKeys * srcK.row_bytes;
    rel_n -= kKeys;
    ++t;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  };
  iteration(IC<1>{}, IC<1>{});
  while (t + 1 < n_full) iteration(IC<0>{}, IC<0>{});   // every wave passes one barrier per iteration in either loop
  while (t < n_tiles) iteration(IC<0>{}, IC<1>{});
  settle();

  // O = O^T / l, through the wave's own LDS area: a lane owns a row's values in pieces of 4 columns, and written as
  // they stand each store instruction would touch 32 rows with 16 bytes each; transposed, a store instruction
  // writes four whole rows.
  LDS_PTR(char) ep = lds + 4 * kTileBytes<D> + wave * kOutBytes;
  constexpr int kChunks = kRowBytes<D> / 16, kRowsPerStore = 64 / kChunks;   // 16-byte chunks per row; rows per store
  const int st_row = lane / kChunks, st_chunk = lane % kChunks;
#pragma unroll
  for (int hb = 0; hb < 2; ++hb) {
    const float l_run = lr[hb] + lu[hb];
    const float l_tot = l_run + xor32(l_run);
    const float inv = 1.f / l_tot;
    const int h = h0 + hb;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = (bf16)(o[hb][db][4 * gq + x] * inv);
        *reinterpret_cast<LDS_PTR(bf16x4)>(ep + l32 * kOutStride + (32 * db + 8 * gq + 4 * half) * 2) = w;
      }
    if (half == 0 && my_row < q_end) lse[(size_t)h * T + my_row] = (m_ref[hb] + __builtin_amdgcn_logf(l_tot)) * kLn2;
#pragma unroll
    for (int j = 0; j < 32 / kRowsPerStore; ++j) {
      const int r = j * kRowsPerStore + st_row;
      const bf16x8 w = *reinterpret_cast<LDS_PTR(const bf16x8)>(ep + r * kOutStride + st_chunk * 16);
      if (q0w + r < q_end) *reinterpret_cast<bf16x8*>(o_out + ((size_t)(q0w + r) * Hq + h) * D + st_chunk * 8) = w;
    }
  }
}

// A block walks the work list in rounds of the grid's size (the launch has as many blocks as the chip holds at
// one per compute unit, a multiple of 8, so a block stays with one residue of the block -> item mapping, i.e.
// with the K/V streams of its XCD).
// The next item's descriptor is fetched while the current item runs -- with a vector load: a scalar load
// in flight would make the hand-counted LDS waits of the tile loop unreliable -- so that an item starts with
// its own loads instead of a chain of dependent ones.
template <int D>
__device__ __forceinline__ void fwd_wide_walk(const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
                                              bf16* __restrict__ o, float* __restrict__ lse, const QItem* __restrict__ items,
                                              int n_items, int T, int Hq, int Hkv, float scale) {
  const int g2 = (Hq / Hkv) >> 1;
  const int total = ((n_items * Hkv + 7) / 8) * 8 * g2;   // block numbers of the mapping, padding included
  const __amdgpu_buffer_rsrc_t irsrc = __builtin_amdgcn_make_buffer_rsrc((void*)items, 0, n_items * (int)sizeof(QItem), 0x00020000);
  typedef __attribute__((__vector_size__(4 * sizeof(int)))) int intx4;
  auto fetch = [&](int b, int* hk, int* hp) -> intx4 {  // block number -> descriptor (zero rows for padding numbers)
    int idx = 0;
    const bool ok = b < total && map_block(b, g2, Hkv, n_items, &idx, hk, hp);
    const intx4 z = {0, 0, 0, 0};
    return ok ? __builtin_bit_cast(intx4, __builtin_amdgcn_raw_buffer_load_b128(irsrc, 0, idx * (int)sizeof(QItem), 0)) : z;
  };
  // round k takes the numbers k G .. k G + G - 1; within its residue class a block goes up the list in even
  // rounds and down in odd ones, which evens out the shares of a list sorted by weight
  const int G = gridDim.x, r8 = blockIdx.x & 7, j8 = blockIdx.x >> 3;
  auto number = [&](int round) -> int { return round * G + ((round & 1) ? 8 * ((G >> 3) - 1 - j8) + r8 : 8 * j8 + r8); };
  int hk = 0, hp = 0, hk_n = 0, hp_n = 0;
  intx4 cur = fetch(number(0), &hk, &hp);
  for (int round = 0; round * G < total; ++round) {
    const intx4 nxt = fetch(number(round + 1), &hk_n, &hp_n);
    QItem it;
    it.q_row0 = __builtin_amdgcn_readfirstlane(cur[0]);
    it.q_rows = __builtin_amdgcn_readfirstlane(cur[1]);
    it.kv_start = __builtin_amdgcn_readfirstlane(cur[2]);
    it.pad = 0;
    if (it.q_rows > 0) fwd_wide_item<D>(it, hk, hp, q, k, v, o, lse, T, Hq, Hkv, scale);
    cur = nxt;
    hk = hk_n;
    hp = hp_n;
  }
}

__global__ __launch_bounds__(256, 1) void fwd_wide_bf16_kernel_d128(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                                     const bf16* __restrict__ v, bf16* __restrict__ o,
                                                                     float* __restrict__ lse, const QItem* __restrict__ items,
                                                                     int n_items, int T, int Hq, int Hkv, float scale) {
  fwd_wide_walk<128>(q, k, v, o, lse, items, n_items, T, Hq, Hkv, scale);
}

}  // namespace

int launch_fwd_wide_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, void* o, float* lse,
                         const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const int g = p.n_q_heads / p.n_kv_heads;
  // one block per compute unit is resident (512 registers per lane); the device's count, rounded to the mapping's 8
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    n_cu = (v + 7) / 8 * 8;
  }
  const int total = mapped_grid(n_items, p.n_kv_heads, g / 2);
  const dim3 grid(total < n_cu ? total : n_cu), block(256);
  // (the body also instantiates at head dim 64, where it is bound by the vector unit and no faster than the
  // two-wave kernel: 1033 against 1027 TFLOP/s on a 16K sample; not dispatched)
  hipLaunchKernelGGL(fwd_wide_bf16_kernel_d128, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                     (const bf16*)v, (bf16*)o, lse, items, n_items, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale);
  return (int)hipGetLastError();
}

}  // namespace slimattn
