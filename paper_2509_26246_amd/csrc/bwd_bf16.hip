// Backward, bf16 inputs, MFMA products with fp32 accumulation.
//
// The scores are recomputed from q, k and the saved lse (paper, Asymmetric Cost Profile: the
// backward of memory-efficient attention re-does the score product, which is why it costs 2.5x
// the forward).  Two kernels:
//   dQ    : a block owns 128 query rows of one head and walks the keys it can see;
//           S^T = K Q^T, dP^T = V dO^T, dS^T = P^T o (dP^T - delta), dQ^T += K^T dS^T.
//   dK/dV : a block owns 128 key rows of one KV head and walks every query row of the launch
//           scope at or after them, for every query head of the group, in a fixed order;
//           S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.  A key tile's gradient is thus
//           summed by its single owner (the paper's "KV gradients from subsequent slices"),
//           with no float atomics; across launches the owner continues from fp32 accumulators.
// In both, the lane layout of the first products' accumulators is, unchanged, the B operand of
// the last products; the matching A operands (K^T, dO^T, Q^T) come from LDS transpose loads.
#include <hip/hip_runtime.h>

#include "internal.h"
#include "mfma_utils.h"

namespace slimattn {
namespace {

constexpr int kDqBQ = 128, kDqBK = 64;
constexpr int kKvOwn = 128, kQStep = 64;
constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void delta_bf16_kernel(const bf16* __restrict__ o, const bf16* __restrict__ dO,
                                                         float* __restrict__ delta, int T, int Hq) {
  constexpr int LPR = D / 8;                                   // lanes per (row, head)
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t rh = idx / LPR;                                // row * Hq + head
  const bool live = rh < (int64_t)T * Hq;
  float s = 0.f;
  if (live) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + idx * 8);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(dO + idx * 8);
#pragma unroll
    for (int t = 0; t < 8; ++t) s = fmaf((float)a[t], (float)b[t], s);
  }
#pragma unroll
  for (int w = LPR / 2; w >= 1; w >>= 1) s += __shfl_xor(s, w);
  if (live && (idx % LPR) == 0) delta[(size_t)(rh % Hq) * T + (rh / Hq)] = s;
}

// ---------------------------------------------------------------------------------------------
// One 64-key tile of the dQ walk for this wave's 32 query rows.  MASKED tiles touch the diagonal.
// pk[ks]: this lane's K-fragment address (key block 0, head-dim step ks) in the current buffer; the
// V tile has the same layout kTileBytes further on.  pkt[db][0..1]: K^T-fragment address pair.
template <int D, bool MASKED>
__device__ __forceinline__ void dq_tile(const lds_cptr (&pk)[D / 16], const lds_cptr (&pkt)[D / 32][2],
                                        const bf16x8 (&qf)[D / 16], const bf16x8 (&dof)[D / 16], floatx16 (&acc)[D / 32],
                                        float lse2, float dlt, int rel) {
  constexpr int NKS = D / 16, NDB = D / 32, kRowBytes = D * 2, kTileBytes = kDqBK * D * 2;
  bf16x8 dsf[4];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    floatx16 sc, dpc;
#pragma unroll
    for (int r = 0; r < 16; ++r) { sc[r] = -lse2; dpc[r] = 0.f; }
    // S^T = K Q^T - lse (log2 units: qf holds q * scale * log2 e) and dP^T = V dO^T for 32 keys:
    // K and V fragments alternate in one stream
    frag_pipeline<2 * NKS, 4, 1, 1>(
        [&](int i) { return lds_ld_row(pk[i >> 1], b * 32 * kRowBytes + (i & 1) * kTileBytes); },
        [&](int i, bf16x8 f) {
          if (i & 1) dpc = mfma32(f, dof[i >> 1], dpc);
          else sc = mfma32(f, qf[i >> 1], sc);
        });
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(sc[r]);
      const float ds = p * (dpc[r] - dlt);
      sc[r] = (MASKED && 32 * b + 8 * (r >> 2) + (r & 3) > rel) ? 0.f : ds;   // key > row contributes nothing
    }
    dsf[2 * b] = pack8(sc, 0);
    dsf[2 * b + 1] = pack8(sc, 8);
  }
  // dQ^T += K^T dS^T, K^T fragments by LDS transpose loads
  frag_pipeline<4 * NDB, 4, 2, 1>(
      [&](int i) { return lds_ld_tr(pkt[i >> 2][0], pkt[i >> 2][1], (i & 3) * 16 * kRowBytes); },
      [&](int i, bf16x8 f) { acc[i >> 2] = mfma32(f, dsf[i & 3], acc[i >> 2]); });
}

template <int D>
__global__ __launch_bounds__(256, 2) void dq_bf16_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                         const bf16* __restrict__ v, const bf16* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dQ, const QItem* __restrict__ items, int n_items,
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
  const TileSource srcK = make_tile_source<D, 256>(k, it.kv_start, Hkv, hk, T, tid);
  const TileSource srcV = make_tile_source<D, 256>(v, it.kv_start, Hkv, hk, T, tid);
  stage_tile<D, kDqBK, 256>(lds, srcK, 0, tid);
  stage_tile<D, kDqBK, 256>(lds + kTileBytes, srcV, 0, tid);

  bf16x8 qf[NKS], dof[NKS];
  {
    const size_t off = ((size_t)ld_row * Hq + h) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      qf[ks] = scale8(*reinterpret_cast<const bf16x8*>(q + off + 16 * ks), scale * kLog2e);
      dof[ks] = *reinterpret_cast<const bf16x8*>(dO + off + 16 * ks);
    }
  }
  const float lse2 = lse[(size_t)h * T + ld_row] * kLog2e;
  const float dlt = delta[(size_t)h * T + ld_row];
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
    // next tile straight into the other buffer (zeros past the end of the tensor; unused then)
    const int nb = ((t + 1) & 1) * kBufBytes;
    stage_tile<D, kDqBK, 256>(lds + nb, srcK, (t + 1) * kDqBK, tid);
    stage_tile<D, kDqBK, 256>(lds + nb + kTileBytes, srcV, (t + 1) * kDqBK, tid);
    const int rel = my_row - j0 - 4 * half;
    if (j0 + kDqBK - 1 <= q0w) {
      dq_tile<D, false>(pk, pkt, qf, dof, acc, lse2, dlt, rel);
    } else if (j0 <= q0w + 31) {
      dq_tile<D, true>(pk, pkt, qf, dof, acc, lse2, dlt, rel);
    }
    const int flip = (t & 1) ? -kBufBytes : kBufBytes;   // fragment addresses follow the buffer switch
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) pk[ks] += flip;
#pragma unroll
    for (int db = 0; db < NDB; ++db) { pkt[db][0] += flip; pkt[db][1] += flip; }
    __builtin_amdgcn_s_waitcnt(0);                 // this thread's direct loads have landed
    __syncthreads();
  }
  if (my_row < q_end) {
    bf16* out = dQ + ((size_t)my_row * Hq + h) * D;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        bf16x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = (bf16)(acc[db][4 * gq + x] * scale);
        *reinterpret_cast<bf16x4*>(out + 32 * db + 8 * gq + 4 * half) = w;
      }
  }
}

// ---------------------------------------------------------------------------------------------
// One 32-row query block against this wave's 32 keys.  MASKED blocks touch the diagonal or the end
// of the query run: rows before the key or at/after q_hi contribute nothing.
// pq[ks]: this lane's Q-fragment address (query block 0, head-dim step ks) in the current buffer;
// the dO tile has the same layout kTileBytes further on.  pqt[db][0..1]: Q^T-fragment address pair.
template <int D, bool MASKED>
__device__ __forceinline__ void dkdv_block(const lds_cptr (&pq)[D / 16], const lds_cptr (&pqt)[D / 32][2],
                                           const float* s_lse, const float* s_delta, int qb, const bf16x8 (&kf)[D / 16],
                                           const bf16x8 (&vf)[D / 16], floatx16 (&dk)[D / 32], floatx16 (&dv)[D / 32],
                                           int rel_lo, int rel_hi, int half) {
  constexpr int NKS = D / 16, NDB = D / 32, kRowBytes = D * 2, kTileBytes = kQStep * D * 2;
  constexpr int kPreRow = D == 128 ? 2 : 4, kPreTr = D == 128 ? 2 : 4;   // read-ahead depth, bounded by registers
  const int qoff = qb * 32 * kRowBytes;
  // S = Q K^T - lse in log2 units (kf holds k * scale * log2 e); the accumulator starts at -lse of
  // its row: local row 32 qb + 8 (r/4) + 4 half + r%4
  floatx16 s;
#pragma unroll
  for (int gq = 0; gq < 4; ++gq) {
    const floatx4 l4 = *reinterpret_cast<const floatx4*>(&s_lse[32 * qb + 8 * gq + 4 * half]);
#pragma unroll
    for (int x = 0; x < 4; ++x) s[4 * gq + x] = -l4[x];
  }
  frag_pipeline<NKS, kPreRow, 1, 1>([&](int i) { return lds_ld_row(pq[i], qoff); },
                                    [&](int i, bf16x8 f) { s = mfma32(f, kf[i], s); });
  // P = exp(S - lse)
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int c = 32 * qb + 8 * (r >> 2) + (r & 3);                 // c + 4*half = local row
    const float p = __builtin_amdgcn_exp2f(s[r]);
    s[r] = (MASKED && (c < rel_lo || c >= rel_hi)) ? 0.f : p;
  }
  const bf16x8 pf0 = pack8(s, 0), pf1 = pack8(s, 8);
  floatx16 dp;
#pragma unroll
  for (int r = 0; r < 16; ++r) dp[r] = 0.f;
  // dP = dO V^T
  frag_pipeline<NKS, kPreRow, 1, 1>([&](int i) { return lds_ld_row(pq[i], qoff + kTileBytes); },
                                    [&](int i, bf16x8 f) { dp = mfma32(f, vf[i], dp); });
#pragma unroll
  for (int gq = 0; gq < 4; ++gq) {
    const floatx4 d4 = *reinterpret_cast<const floatx4*>(&s_delta[32 * qb + 8 * gq + 4 * half]);
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int r = 4 * gq + x;
      dp[r] = s[r] * (dp[r] - d4[x]);                                // dS = P (dP - delta)
    }
  }
  const bf16x8 dsf0 = pack8(dp, 0), dsf1 = pack8(dp, 8);
  // dV^T += dO^T P and dK^T += Q^T dS: transposed dO and Q fragments alternate in one stream
  frag_pipeline<4 * NDB, kPreTr, 2, 1>(
      [&](int i) {
        const int off = qoff + ((i >> 1) & 1) * 16 * kRowBytes + ((i & 1) ? 0 : kTileBytes);
        return lds_ld_tr(pqt[i >> 2][0], pqt[i >> 2][1], off);
      },
      [&](int i, bf16x8 f) {
        const int db = i >> 2, ks = (i >> 1) & 1;
        if (i & 1) dk[db] = mfma32(f, ks ? dsf1 : dsf0, dk[db]);
        else dv[db] = mfma32(f, ks ? pf1 : pf0, dv[db]);
      });
}

template <int D>
__global__ __launch_bounds__(256, 2) void dkdv_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v, const bf16* __restrict__ dO,
    const float* __restrict__ lse, const float* __restrict__ delta, float* __restrict__ acc_dk, float* __restrict__ acc_dv,
    bf16* __restrict__ dK, bf16* __restrict__ dV, const KvItem* __restrict__ items, int n_items, const Seg* __restrict__ segs,
    int T, int Hq, int Hkv, float scale, int load_acc, int store_final) {
  constexpr int NKS = D / 16, NDB = D / 32;
  constexpr int kTileBytes = kQStep * D * 2, kBufBytes = 2 * kTileBytes;
  __shared__ __attribute__((aligned(1024))) char smem[2 * kBufBytes];   // [buffer][Q tile, dO tile]
  __shared__ __attribute__((aligned(16))) float s_lse[2][kQStep];
  __shared__ __attribute__((aligned(16))) float s_delta[2][kQStep];

  const int g = Hq / Hkv;
  // one block per (key tile, kv head); kv heads of one tile adjacent, heavy tiles first
  const int item_idx = blockIdx.x / Hkv, hk = blockIdx.x % Hkv;
  if (item_idx >= n_items) return;
  const KvItem it = items[item_idx];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int kv0w = it.kv_row0 + 32 * wave, my_key = kv0w + l32, kv_end = it.kv_row0 + it.kv_rows;
  const int ld_key = min(my_key, T - 1);
  LDS_PTR(char) lds = (LDS_PTR(char))smem;

  // Flattened walk: for each run, for each head of the group, for each 64-row step.  Rows are
  // addressed relative to the key tile's first row (every run of the item lies at or after it).
  int sgi = it.seg_begin, hh = 0;
  Seg sg = segs[sgi];
  int i0 = max(sg.q_lo, it.kv_row0);
  bool have = true;                                   // a key tile always has at least its own rows
  const TileSource srcQ = make_tile_source<D, 256>(q, it.kv_row0, Hq, 0, T, tid);
  const TileSource srcDO = make_tile_source<D, 256>(dO, it.kv_row0, Hq, 0, T, tid);
  const int head_bytes = D * 2;
#define SLIMATTN_STAGE(buf_, row0_, head_)                                                                     \
  do {                                                                                                         \
    TileSource a_ = srcQ, b_ = srcDO;                                                                          \
    a_.voff += (head_) * head_bytes;                                                                           \
    b_.voff += (head_) * head_bytes;                                                                           \
    stage_tile<D, kQStep, 256>(lds + (buf_) * kBufBytes, a_, (row0_) - it.kv_row0, tid);                       \
    stage_tile<D, kQStep, 256>(lds + (buf_) * kBufBytes + kTileBytes, b_, (row0_) - it.kv_row0, tid);          \
    if (tid < kQStep) {                                                                                        \
      const int r_ = min((row0_) + tid, T - 1);                                                                \
      s_lse[(buf_)][tid] = lse[(size_t)(head_) * T + r_] * kLog2e;                                             \
      s_delta[(buf_)][tid] = delta[(size_t)(head_) * T + r_];                                                  \
    }                                                                                                          \
  } while (0)
  SLIMATTN_STAGE(0, i0, hk * g + hh);

  bf16x8 kf[NKS], vf[NKS];
  {
    const size_t off = ((size_t)ld_key * Hkv + hk) * D + 8 * half;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      kf[ks] = scale8(*reinterpret_cast<const bf16x8*>(k + off + 16 * ks), scale * kLog2e);
      vf[ks] = *reinterpret_cast<const bf16x8*>(v + off + 16 * ks);
    }
  }
  lds_cptr pq[NKS], pqt[NDB][2];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) pq[ks] = lds_row_ptr<D>(lds, l32, 16 * ks + 8 * half);
#pragma unroll
  for (int db = 0; db < NDB; ++db) lds_tr_ptrs<D>(lds, 32 * db, lane, pqt[db][0], pqt[db][1]);
  floatx16 dk[NDB], dv[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[db][r] = 0.f; dv[db][r] = 0.f; }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  int buf = 0;
  while (have) {
    const int cur_i0 = i0, cur_hi = sg.q_hi;
    // advance to the next step (uniform across the block) and start fetching it
    i0 += kQStep;
    if (i0 >= sg.q_hi) {
      if (++hh == g) {
        hh = 0;
        if (++sgi == it.seg_end) have = false; else sg = segs[sgi];
      }
      if (have) i0 = max(sg.q_lo, it.kv_row0);
    }
    if (have) SLIMATTN_STAGE(buf ^ 1, i0, hk * g + hh);

    // local rows [rel_lo, rel_hi) minus 4*half contribute: row >= key and row < end of the run
    const int rel_lo = my_key - cur_i0 - 4 * half, rel_hi = cur_hi - cur_i0 - 4 * half;
#pragma unroll
    for (int qb = 0; qb < kQStep / 32; ++qb) {
      const int r0 = cur_i0 + 32 * qb;               // first row of the block
      if (r0 + 31 < kv0w || r0 >= cur_hi) continue;  // wave-uniform: nothing at or after the wave's keys
      if (r0 >= kv0w + 31 && r0 + 32 <= cur_hi)
        dkdv_block<D, false>(pq, pqt, s_lse[buf], s_delta[buf], qb, kf, vf, dk, dv, rel_lo, rel_hi, half);
      else
        dkdv_block<D, true>(pq, pqt, s_lse[buf], s_delta[buf], qb, kf, vf, dk, dv, rel_lo, rel_hi, half);
    }
    const int flip = buf ? -kBufBytes : kBufBytes;   // fragment addresses follow the buffer switch
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) pq[ks] += flip;
#pragma unroll
    for (int db = 0; db < NDB; ++db) { pqt[db][0] += flip; pqt[db][1] += flip; }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    buf ^= 1;
  }
#undef SLIMATTN_STAGE

  if (my_key < kv_end) {
    const size_t base = ((size_t)my_key * Hkv + hk) * D;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const size_t off = base + 32 * db + 8 * gq + 4 * half;
        floatx4 a, b;
#pragma unroll
        for (int x = 0; x < 4; ++x) { a[x] = dk[db][4 * gq + x] * scale; b[x] = dv[db][4 * gq + x]; }
        if (load_acc) {
          const floatx4 pa = *reinterpret_cast<const floatx4*>(acc_dk + off);
          const floatx4 pb = *reinterpret_cast<const floatx4*>(acc_dv + off);
          a += pa;
          b += pb;
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

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ a, bf16* __restrict__ b, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const floatx4 x = reinterpret_cast<const floatx4*>(a)[i];
  bf16x4 w;
#pragma unroll
  for (int t = 0; t < 4; ++t) w[t] = (bf16)x[t];
  reinterpret_cast<bf16x4*>(b)[i] = w;
}

}  // namespace

int dq_q_tile(int dtype, int) { return dtype == SLIMATTN_F32 ? 64 : kDqBQ; }
int dkdv_kv_tile(int dtype, int) { return dtype == SLIMATTN_F32 ? 64 : kKvOwn; }

int launch_bwd_delta_bf16(const LaunchCtx& c, const void* o, const void* dO, float* delta) {
  const slimattn_params& p = *c.p;
  const int64_t n = c.T * p.n_q_heads * (p.head_dim / 8);
  if (n == 0) return 0;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(delta_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)o, (const bf16*)dO, delta,
                       (int)c.T, p.n_q_heads);
  else
    hipLaunchKernelGGL(delta_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)o, (const bf16*)dO, delta,
                       (int)c.T, p.n_q_heads);
  return (int)hipGetLastError();
}

int launch_bwd_dq_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, const void* dO, const float* lse,
                       const float* delta, void* dQ, const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const int g = p.n_q_heads / p.n_kv_heads;
  const dim3 grid(mapped_grid(n_items, p.n_kv_heads, g)), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(dq_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, lse, delta, (bf16*)dQ, items, n_items, (int)c.T, p.n_q_heads,
                       p.n_kv_heads, p.scale);
  else
    hipLaunchKernelGGL(dq_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, lse, delta, (bf16*)dQ, items, n_items, (int)c.T, p.n_q_heads,
                       p.n_kv_heads, p.scale);
  return (int)hipGetLastError();
}

int launch_bwd_dkdv_bf16(const LaunchCtx& c, const void* q, const void* k, const void* v, const void* dO, const float* lse,
                         const float* delta, float* acc_dk, float* acc_dv, void* dK, void* dV, const KvItem* items,
                         int n_items, const Seg* segs, int load_acc, int store_final) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  const dim3 grid((unsigned)(n_items * p.n_kv_heads)), block(256);
  if (p.head_dim == 128)
    hipLaunchKernelGGL(dkdv_bf16_kernel<128>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, lse, delta, acc_dk, acc_dv, (bf16*)dK, (bf16*)dV, items, n_items,
                       segs, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale, load_acc, store_final);
  else
    hipLaunchKernelGGL(dkdv_bf16_kernel<64>, grid, block, 0, (hipStream_t)c.stream, (const bf16*)q, (const bf16*)k,
                       (const bf16*)v, (const bf16*)dO, lse, delta, acc_dk, acc_dv, (bf16*)dK, (bf16*)dV, items, n_items,
                       segs, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale, load_acc, store_final);
  return (int)hipGetLastError();
}

int launch_finalize_bf16(const LaunchCtx& c, const float* acc_dk, const float* acc_dv, void* dK, void* dV) {
  const slimattn_params& p = *c.p;
  const int64_t n4 = c.T * p.n_kv_heads * p.head_dim / 4;
  if (n4 == 0) return 0;
  const dim3 grid((unsigned)((n4 + 255) / 256)), block(256);
  hipLaunchKernelGGL(cast_bf16_kernel, grid, block, 0, (hipStream_t)c.stream, acc_dk, (bf16*)dK, n4);
  hipLaunchKernelGGL(cast_bf16_kernel, grid, block, 0, (hipStream_t)c.stream, acc_dv, (bf16*)dV, n4);
  return (int)hipGetLastError();
}

}  // namespace slimattn
