// Backward, bf16 inputs, MFMA products with fp32 accumulation.
//
// The scores are recomputed from q, k and the saved lse (paper, Asymmetric Cost Profile: the
// backward of memory-efficient attention re-does the score product, which is why it costs 2.5x
// the forward).  Two kernels:
//   dQ    : a block owns 128 query rows of one head and walks the keys it can see;
//           S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T.
//   dK/dV : (dkdv_wide_bf16.hip) a block owns 256 key rows of one KV head and walks every query row of
//           the launch scope at or after them, for every query head of the group, in a fixed order;
//           S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.  A key tile's gradient, which collects
//           from every later slice of its sample (the inter-slice dependency of the backward pass in the
//           paper's DAG simulator section), is thus summed by its single owner, with no float atomics;
//           across launches the owner continues from fp32 accumulators.
// In both, the lane layout of the first products' accumulators is, unchanged, the B operand of
// the last products; the matching A operands (K^T, dO^T, Q^T) come from LDS transpose loads.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "mfma_utils.h"

namespace slimattn {
namespace {

constexpr int kDqBQ = 128, kDqBK = 64;
constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------
// x as three bf16 terms (w[at], w[at + 1], w[at + 2]) whose sum is x to fp32 precision
__device__ __forceinline__ void split3(float x, bf16x8& w, int at) {
  const bf16 a = (bf16)x;
  float r = x - (float)a;
  const bf16 b = (bf16)r;
  r -= (float)b;
  w[at] = a;
  w[at + 1] = b;
  w[at + 2] = (bf16)r;
}

// Two bf16 triples of a row's statistics: -lse2 in elements 0..2, -delta in 4..6.
__device__ __forceinline__ bf16x8 stat_triples(float lse2, float dlt) {
  bf16x8 w;
  split3(-lse2, w, 0);
  split3(-dlt, w, 4);
  w[3] = (bf16)0.f;
  w[7] = (bf16)0.f;
  return w;
}

// Prepass: the statistics of the query rows of the listed tiles, every head (launches whose dQ kernel does not
// compute them itself).  grid = (tiles, kStatSplit); D / 8 lanes share a (row, head).
constexpr int kStatSplit = 4;
template <int D>
__global__ __launch_bounds__(256) void stat_bf16_kernel(const bf16* __restrict__ o, const bf16* __restrict__ dO,
                                                        const float* __restrict__ lse, bf16x8* __restrict__ stat3,
                                                        const QItem* __restrict__ items, int T, int Hq) {
  constexpr int LPR = D / 8;                                   // lanes per (row, head)
  const QItem it = items[blockIdx.x];
  const int n = it.q_rows * Hq * LPR;                          // lane tasks of the tile: a multiple of LPR
  // every lane of a group of LPR runs the same iterations (the stride is a multiple of 64), so the
  // shuffles below always see the whole group
  for (int e0 = blockIdx.y * 256; e0 < n; e0 += kStatSplit * 256) {
    const int e = e0 + threadIdx.x;
    const bool live = e < n;
    const int rh = live ? e / LPR : 0;                         // local row * Hq + head
    const int row = it.q_row0 + rh / Hq, h = rh % Hq;
    float s = 0.f;
    if (live) {
      const size_t at = ((size_t)row * Hq + h) * D + (size_t)(e % LPR) * 8;
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + at);
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(dO + at);
#pragma unroll
      for (int t = 0; t < 8; ++t) s = fmaf((float)a[t], (float)b[t], s);
    }
#pragma unroll
    for (int w = LPR / 2; w >= 1; w >>= 1) s += __shfl_xor(s, w);
    if (live && (e % LPR) == 0) {
      const size_t at = (size_t)h * T + row;
      stat3[at] = stat_triples(lse[at] * kLog2e, s);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// One 64-key tile of the dQ walk for this wave's 32 query rows.  MASKED tiles touch the diagonal.
// pk[ks]: this lane's K-fragment address (key block 0, head-dim step ks) in the current buffer; the
// V tile has the same layout kTileBytes further on.  pkt[db][0..1]: K^T-fragment address pair.
template <int D, bool MASKED>
__device__ __forceinline__ void dq_tile(const lds_cptr (&pk)[D / 16], const lds_cptr (&pkt)[D / 32][2],
                                        const bf16x8 (&qf)[D / 16], const bf16x8 (&dof)[D / 16], floatx16 (&acc)[D / 32],
                                        const floatx16& negl, const floatx16& negd, int rel) {
  constexpr int NKS = D / 16, NDB = D / 32, kRowBytes = D * 2, kTileBytes = kDqBK * D * 2;
  bf16x8 dsf[4];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    floatx16 sc, dpc;
    // S^T = K Q^T - lse (log2 units: qf holds q * scale * log2 e) and dP^T = V dO^T - delta for 32 keys: K and V
    // fragments alternate in one stream.  The first product of each accumulator takes its C operand from a
    // register block that holds -lse (-delta) of the lane's row in every register: nothing is initialised and
    // the element-wise part has no subtraction.
    frag_pipeline<2 * NKS, 4, 1, 1>(
        [&](int i) { return lds_ld_row(pk[i >> 1], b * 32 * kRowBytes + (i & 1) * kTileBytes); },
        [&](int i, bf16x8 f) {
          if (i & 1) dpc = mfma32(f, dof[i >> 1], i == 1 ? negd : dpc);
          else sc = mfma32(f, qf[i >> 1], i == 0 ? negl : sc);
        });
    // the element-wise part runs at raised priority: a wave that streams products would otherwise
    // keep the vector issue port and starve the other wave's softmax
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(sc[r]);
      const float ds = p * dpc[r];
      sc[r] = (MASKED && 32 * b + 8 * (r >> 2) + (r & 3) > rel) ? 0.f : ds;   // key > row contributes nothing
    }
    dsf[2 * b] = pack8(sc, 0);
    dsf[2 * b + 1] = pack8(sc, 8);
    __builtin_amdgcn_s_setprio(0);
  }
  // dQ^T += K^T dS^T: one batch of K^T fragments per 16-key step j (one fragment per head-dim block), so that
  // consecutive products go to different accumulators (a product on the accumulator of the one right
  // before it has to wait for that one's result)
  constexpr int kStep = 16 * kRowBytes;
  if constexpr (NDB == 4) {
    Tr4 tb[4];
    auto issue = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      static_for<0, NDB>([&](auto dc) {
        constexpr int db = decltype(dc)::value;
        tr1_issue<j * kStep>(pkt[db][0], tb[j].r[2 * db]);
        tr1_issue<j * kStep>(pkt[db][1], tb[j].r[2 * db + 1]);
      });
    };
    issue(IC<0>{});
    static_for<0, 4>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      if constexpr (j + 1 < 4) issue(IC<j + 1>{});
      tr4_wait_n<(j + 1 < 4) ? 8 : 0>(tb[j]);
#pragma unroll
      for (int db = 0; db < NDB; ++db) acc[db] = mfma32(tr4_frag(tb[j], db), dsf[j], acc[db]);
    });
  } else {
    Tr2 tb[4];
    auto issue = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      static_for<0, NDB>([&](auto dc) {
        constexpr int db = decltype(dc)::value;
        tr1_issue<j * kStep>(pkt[db][0], tb[j].r[2 * db]);
        tr1_issue<j * kStep>(pkt[db][1], tb[j].r[2 * db + 1]);
      });
    };
    issue(IC<0>{});
    static_for<0, 4>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      if constexpr (j + 1 < 4) issue(IC<j + 1>{});
      lds_wait<(j + 1 < 4) ? 4 : 0>(tb[j]);
#pragma unroll
      for (int db = 0; db < NDB; ++db) acc[db] = mfma32(tr2_frag(tb[j], db), dsf[j], acc[db]);
    });
  }
}

template <int D, bool OWN_STATS>
__global__ __launch_bounds__(256, 2) void dq_bf16_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                         const bf16* __restrict__ v, const bf16* __restrict__ dO,
                                                         const bf16* __restrict__ o, const float* __restrict__ lse,
                                                         bf16x8* __restrict__ stat3, bf16* __restrict__ dQ,
                                                         const QItem* __restrict__ items, int n_items,
                                                         int T, int Hq, int Hkv, float scale) {
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int kTileBytes = kDqBK * D * 2, kBufBytes = 2 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char smem[2 * kBufBytes];   // [buffer][K tile, V tile]

  const int g = Hq / Hkv;
  int item_idx, hk, hg;
  if (!map_block(blockIdx.x, g, Hkv, n_items, &item_idx, &hk, &hg)) return;
  const int h = hk * g + hg;
  const QItem it = items[item_idx];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int q0w = it.q_row0 + 32 * wave, my_row = q0w + l32, q_end = it.q_row0 + it.q_rows;
  const int ld_row = min(my_row, T - 1);
  LDS_PTR(char) lds = (LDS_PTR(char))smem;
  const TileSource srcK = make_tile_source<D, 256>(k, it.kv_start, Hkv, hk, q_end, tid);
  const TileSource srcV = make_tile_source<D, 256>(v, it.kv_start, Hkv, hk, q_end, tid);
  stage_tile<D, kDqBK, 256>(lds, srcK, 0, tid);
  stage_tile<D, kDqBK, 256>(lds + kTileBytes, srcV, 0, tid);

  // The block's Q and dO rows and the row statistics of the backward pass: lse in log2 units and delta =
  // dO . O.  OWN_STATS: computed here (the lane's half of the head dim, then the two half-waves that
  // share a row) and, as every (row, head) of the launch scope belongs to exactly one dQ block, stored for
  // the dK/dV kernel, which runs after this one: -lse2 and -delta as three bf16 terms each (a product
  // with a fragment of ones adds them into an accumulator exactly).  Otherwise a prepass has stored them
  // and the triples are added up again.
  bf16x8 qf[NKS], dof[NKS];
  float dlt = 0.f, lse2;
  {
    const size_t off = ((size_t)ld_row * Hq + h) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      qf[ks] = scale8(*reinterpret_cast<const bf16x8*>(q + off + 16 * ks), scale * kLog2e);
      dof[ks] = *reinterpret_cast<const bf16x8*>(dO + off + 16 * ks);
      if constexpr (OWN_STATS) {
        const bf16x8 of = *reinterpret_cast<const bf16x8*>(o + off + 16 * ks);
#pragma unroll
        for (int e = 0; e < 4; ++e) {                   // packed bf16 pairs, fp32 sum
          const bf16x2 a2 = {of[2 * e], of[2 * e + 1]}, b2 = {dof[ks][2 * e], dof[ks][2 * e + 1]};
          dlt = __builtin_amdgcn_fdot2_f32_bf16(a2, b2, dlt, false);
        }
      }
    }
  }
  if constexpr (OWN_STATS) {
    dlt += xor32(dlt);
    lse2 = lse[(size_t)h * T + ld_row] * kLog2e;
    if (half == 0 && my_row < q_end) stat3[(size_t)h * T + my_row] = stat_triples(lse2, dlt);
  } else {
    const bf16x8 w = stat3[(size_t)h * T + ld_row];
    lse2 = -(((float)w[0] + (float)w[1]) + (float)w[2]);
    dlt = -(((float)w[4] + (float)w[5]) + (float)w[6]);
  }
  floatx16 negl, negd;                                  // the C operands of every tile's first products
#pragma unroll
  for (int r = 0; r < 16; ++r) { negl[r] = -lse2; negd[r] = -dlt; }
  asm volatile("" : "+v"(negl), "+v"(negd));            // kept in registers, not rebuilt at every use
  lds_cptr pk[NKS], pkt[NDB][2];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) pk[ks] = lds_row_ptr<D>(lds, l32, 16 * ks + 8 * half);
#pragma unroll
  for (int db = 0; db < NDB; ++db) lds_tr_ptrs<D>(lds, 32 * db, lane, pkt[db][0], pkt[db][1]);
  floatx16 acc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  const int n_tiles = (q_end - it.kv_start + kDqBK - 1) / kDqBK;
  __builtin_amdgcn_s_waitcnt(0);                   // tile 0 has landed in LDS
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = it.kv_start + t * kDqBK;
    // next tile straight into the other buffer (not behind the last one: the wait that ends the iteration would
    // sit out the latency of loads nobody needs)
    const int nb = ((t + 1) & 1) * kBufBytes;
    if (t + 1 < n_tiles) {
      stage_tile<D, kDqBK, 256>(lds + nb, srcK, (t + 1) * kDqBK, tid);
      stage_tile<D, kDqBK, 256>(lds + nb + kTileBytes, srcV, (t + 1) * kDqBK, tid);
    }
    const int rel = my_row - j0 - 4 * half;
    if (j0 + kDqBK - 1 <= q0w) {
      dq_tile<D, false>(pk, pkt, qf, dof, acc, negl, negd, rel);
    } else if (j0 <= q0w + 31) {
      dq_tile<D, true>(pk, pkt, qf, dof, acc, negl, negd, rel);
    }
    const int flip = (t & 1) ? -kBufBytes : kBufBytes;   // fragment addresses follow the buffer switch
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) pk[ks] += flip;
#pragma unroll
    for (int db = 0; db < NDB; ++db) { pkt[db][0] += flip; pkt[db][1] += flip; }
    __builtin_amdgcn_s_waitcnt(0);                 // this thread's direct loads have landed
    __syncthreads();
  }
  // dQ rows out through LDS (the tile buffers are free behind the loop's last barrier; each wave uses a part of
  // its own): a lane owns a row's values in pieces of 4 columns, and written as they stand each store instruction
  // would touch 32 rows with 16 bytes each; transposed, a store instruction writes whole rows.
  constexpr int kOutStride = D * 2 + 16, kChunks = D * 2 / 16, kRowsPerStore = 64 / kChunks;
  static_assert(4 * 32 * kOutStride <= 2 * kBufBytes, "the transposition areas must fit the tile buffers");
  LDS_PTR(char) ep = lds + (tid >> 6) * 32 * kOutStride;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      bf16x4 w;
#pragma unroll
      for (int x = 0; x < 4; ++x) w[x] = (bf16)(acc[db][4 * gq + x] * scale);
      *reinterpret_cast<LDS_PTR(bf16x4)>(ep + l32 * kOutStride + (32 * db + 8 * gq + 4 * half) * 2) = w;
    }
  const int st_row = lane / kChunks, st_chunk = lane % kChunks;
#pragma unroll
  for (int j = 0; j < 32 / kRowsPerStore; ++j) {
    const int r = j * kRowsPerStore + st_row;
    const bf16x8 w = *reinterpret_cast<LDS_PTR(const bf16x8)>(ep + r * kOutStride + st_chunk * 16);
    if (q0w + r < q_end) *reinterpret_cast<bf16x8*>(dQ + ((size_t)(q0w + r) * Hq + h) * D + st_chunk * 8) = w;
  }
}

// ---------------------------------------------------------------------------------------------
// Sum of the partial tiles of a divided key tile, in slot order (fixed, so the result does not
// depend on which block finished first), added to the fp32 accumulators or written as bf16.
// grid = (tiles x kv heads, kReduceSplit): a block takes a 1/kReduceSplit share of the tile's elements
// (the launches are small, and few blocks with long dependent loops would only wait on memory);
// a thread owns four consecutive columns of a row.
constexpr int kReduceSplit = 16;
template <int D>
__global__ __launch_bounds__(256) void reduce_parts_kernel(const float* __restrict__ parts, float* __restrict__ acc_dk,
                                                           float* __restrict__ acc_dv, bf16* __restrict__ dK,
                                                           bf16* __restrict__ dV, const KvReduce* __restrict__ items,
                                                           int Hkv, int tile_rows) {
  const KvReduce it = items[blockIdx.x / Hkv];
  const int hk = blockIdx.x % Hkv;
  const int kTile = tile_rows * D;                     // elements of one partial dK (or dV) tile
  for (int e = (blockIdx.y * 256 + threadIdx.x) * 4; e < 2 * kTile; e += kReduceSplit * 256 * 4) {
    const int which = e / kTile, r = (e % kTile) / D, c = e % D;
    if (r >= it.kv_rows) continue;
    floatx4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < it.n_parts; ++p)
      sum += *reinterpret_cast<const floatx4*>(parts + ((size_t)(it.first_slot + p) * Hkv + hk) * (2 * kTile) + e);
    const size_t off = ((size_t)(it.kv_row0 + r) * Hkv + hk) * D + c;
    float* acc = which ? acc_dv : acc_dk;
    const bool load_acc = it.kv_row0 + r < it.load_until, store_final = it.kv_row0 + r >= it.final_from;
    if (load_acc) sum += *reinterpret_cast<const floatx4*>(acc + off);
    if (store_final) {
      bf16x4 w;
#pragma unroll
      for (int x = 0; x < 4; ++x) w[x] = (bf16)sum[x];
      *reinterpret_cast<bf16x4*>((which ? dV : dK) + off) = w;
    } else {
      *reinterpret_cast<floatx4*>(acc + off) = sum;
    }
  }
}

}  // namespace

int dq_q_tile(int dtype, int) { return dtype == SLIMATTN_F32 ? 64 : kDqBQ; }
int dkdv_kv_tile(int dtype, int) { return dtype == SLIMATTN_F32 ? 64 : kSplitTileRows[0]; }   // bf16: the dK/dV kernel's 256 key rows per block

int launch_bwd_stat_bf16(const LaunchCtx& c, const void* o, const void* dO, const float* lse, void* stat3, const QItem* items,
                         int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const dim3 grid((unsigned)n_items, kStatSplit), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(stat_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)o, (const bf16*)dO, lse,
                       (bf16x8*)stat3, items, (int)c.T, p.n_q_heads);
  else
    hipLaunchKernelGGL(stat_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)o, (const bf16*)dO, lse,
                       (bf16x8*)stat3, items, (int)c.T, p.n_q_heads);
  return (int)hipGetLastError();
}

namespace {
template <int D, bool OWN>
void launch_dq(const LaunchCtx& c, dim3 grid, dim3 block, const void* q, const void* k, const void* v, const void* dO, const void* o,
               const float* lse, void* stat3, void* dQ, const QItem* items, int n_items) {
  const slimattn_params& p = *c.p;
  hipLaunchKernelGGL((dq_bf16_kernel<D, OWN>), grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                     (const bf16*)v, (const bf16*)dO, (const bf16*)o, lse, (bf16x8*)stat3, (bf16*)dQ, items, n_items, (int)c.T,
                     p.n_q_heads, p.n_kv_heads, p.scale);
}
}  // namespace

int launch_bwd_dq_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, const void* dO, const void* o,
                       const float* lse, void* stat3, int own_stats, void* dQ, const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const int g = p.n_q_heads / p.n_kv_heads;
  const dim3 grid(mapped_grid(n_items, p.n_kv_heads, g)), block(256);
  if (p.head_dim == 128) {
    if (own_stats) launch_dq<128, true>(c, grid, block, q, k, v, dO, o, lse, stat3, dQ, items, n_items);
    else launch_dq<128, false>(c, grid, block, q, k, v, dO, o, lse, stat3, dQ, items, n_items);
  } else {
    if (own_stats) launch_dq<64, true>(c, grid, block, q, k, v, dO, o, lse, stat3, dQ, items, n_items);
    else launch_dq<64, false>(c, grid, block, q, k, v, dO, o, lse, stat3, dQ, items, n_items);
  }
  return (int)hipGetLastError();
}

int launch_bwd_reduce_bf16(const LaunchCtx& c, const float* parts, float* acc_dk, float* acc_dv, void* dK, void* dV,
                           const KvReduce* items, int n_items, int tile_rows) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const dim3 grid((unsigned)(n_items * p.n_kv_heads), kReduceSplit), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(reduce_parts_kernel<128>, grid, block, 0, (hipStream_t)c.stream, parts, acc_dk, acc_dv, (bf16*)dK,
                       (bf16*)dV, items, p.n_kv_heads, tile_rows);
  else
    hipLaunchKernelGGL(reduce_parts_kernel<64>, grid, block, 0, (hipStream_t)c.stream, parts, acc_dk, acc_dv, (bf16*)dK,
                       (bf16*)dV, items, p.n_kv_heads, tile_rows);
  return (int)hipGetLastError();
}

}  // namespace slimattn
