// fp32 kernels: plain FMA arithmetic, accurate expf/logf, fixed summation order.  This is the
// "fp32 mode" whose results must agree with the fp64 definition to 1e-5; it is kept separate from
// the MFMA kernels on purpose so that no reduced-precision step can leak into it.
//
// Forward (paper: slice-level causal attention with a KV cache): one lane owns one query row and
// walks the sample's keys kv_start .. row in tiles staged through LDS, keeping a running maximum
// and sum (online softmax).  Backward (paper: scores are recomputed in the backward pass):
// dQ mirrors the forward walk; dK/dV has one owner per key row that walks the query rows at or
// after it, so contributions from later slices are summed in a fixed order without atomics.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace slimattn {
namespace {

constexpr int kRowsF32 = 64;    // query rows per block in fwd / dQ (one per lane)
constexpr int kKeysStage = 32;  // keys staged in LDS per step
constexpr int kKvOwnF32 = 64;   // key rows owned by a dK/dV block (two lanes per row)
constexpr int kQStage = 16;     // query rows staged per step in dK/dV

template <int D>
__global__ __launch_bounds__(kRowsF32) void fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                           const float* __restrict__ v, float* __restrict__ o,
                                                           float* __restrict__ lse, const QItem* __restrict__ items,
                                                           int T, int Hq, int Hkv, float scale) {
  __shared__ float sK[kKeysStage][D];
  __shared__ float sV[kKeysStage][D];
  const QItem it = items[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x;
  const bool live = lane < it.q_rows;
  const int row = min(it.q_row0 + lane, T - 1);
  float qr[D], acc[D];
  const float* qp = q + ((size_t)row * Hq + h) * D;
#pragma unroll
  for (int c = 0; c < D; ++c) { qr[c] = qp[c]; acc[c] = 0.f; }
  float m = -INFINITY, l = 0.f;
  const int kv_end = it.q_row0 + it.q_rows;
  for (int j0 = it.kv_start; j0 < kv_end; j0 += kKeysStage) {
    __syncthreads();
    for (int e = lane; e < kKeysStage * (D / 4); e += kRowsF32) {
      const int r = e / (D / 4), c4 = e % (D / 4);
      // rows from kv_end on belong to other units (their K/V may not exist yet): staged as zeros, so that
      // their probability 0 times their value is 0 whatever the memory holds
      const bool in = j0 + r < kv_end;
      const int jr = min(j0 + r, kv_end - 1);
      const float4 zero = {0.f, 0.f, 0.f, 0.f};
      reinterpret_cast<float4*>(&sK[r][0])[c4] = in ? reinterpret_cast<const float4*>(k + ((size_t)jr * Hkv + hk) * D)[c4] : zero;
      reinterpret_cast<float4*>(&sV[r][0])[c4] = in ? reinterpret_cast<const float4*>(v + ((size_t)jr * Hkv + hk) * D)[c4] : zero;
    }
    __syncthreads();
    float s[kKeysStage];
    float tile_max = -INFINITY;
#pragma unroll
    for (int r = 0; r < kKeysStage; ++r) {
      float d0 = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) d0 = fmaf(qr[c], sK[r][c], d0);
      s[r] = (j0 + r <= row) ? d0 * scale : -INFINITY;
      tile_max = fmaxf(tile_max, s[r]);
    }
    const float m_new = fmaxf(m, tile_max);           // finite: key j0 <= row always holds for live rows
    const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
    l *= alpha;
#pragma unroll
    for (int c = 0; c < D; ++c) acc[c] *= alpha;
#pragma unroll
    for (int r = 0; r < kKeysStage; ++r) {
      const float p = (s[r] == -INFINITY) ? 0.f : expf(s[r] - m_new);
      l += p;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(p, sV[r][c], acc[c]);
    }
    m = m_new;
  }
  if (live) {
    const float inv = 1.f / l;
    float* op = o + ((size_t)row * Hq + h) * D;
#pragma unroll
    for (int c = 0; c < D; ++c) op[c] = acc[c] * inv;
    lse[(size_t)h * T + row] = m + logf(l);
  }
}

// delta = rowsum(dO * O) for the query rows of the listed tiles and every head: one block per tile.
template <int D>
__global__ __launch_bounds__(256) void delta_f32_kernel(const float* __restrict__ o, const float* __restrict__ dO,
                                                        float* __restrict__ delta, const QItem* __restrict__ items, int T,
                                                        int Hq) {
  const QItem it = items[blockIdx.x];
  for (int e = threadIdx.x; e < it.q_rows * Hq; e += 256) {
    const int row = it.q_row0 + e / Hq, h = e % Hq;
    const float* a = o + ((size_t)row * Hq + h) * D;
    const float* b = dO + ((size_t)row * Hq + h) * D;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < D; ++c) s = fmaf(a[c], b[c], s);
    delta[(size_t)h * T + row] = s;
  }
}

template <int D>
__global__ __launch_bounds__(kRowsF32) void dq_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                          const float* __restrict__ v, const float* __restrict__ dO,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          float* __restrict__ dQ, const QItem* __restrict__ items, int T,
                                                          int Hq, int Hkv, float scale) {
  __shared__ float sK[kKeysStage][D];
  __shared__ float sV[kKeysStage][D];
  const QItem it = items[blockIdx.x];
  const int h = blockIdx.y, hk = h / (Hq / Hkv);
  const int lane = threadIdx.x;
  const bool live = lane < it.q_rows;
  const int row = min(it.q_row0 + lane, T - 1);
  float qr[D], dor[D], acc[D];
  const float* qp = q + ((size_t)row * Hq + h) * D;
  const float* dp_ = dO + ((size_t)row * Hq + h) * D;
#pragma unroll
  for (int c = 0; c < D; ++c) { qr[c] = qp[c]; dor[c] = dp_[c]; acc[c] = 0.f; }
  const float row_lse = lse[(size_t)h * T + row], row_delta = delta[(size_t)h * T + row];
  const int kv_end = it.q_row0 + it.q_rows;
  for (int j0 = it.kv_start; j0 < kv_end; j0 += kKeysStage) {
    __syncthreads();
    for (int e = lane; e < kKeysStage * (D / 4); e += kRowsF32) {
      const int r = e / (D / 4), c4 = e % (D / 4);
      const int jr = min(j0 + r, T - 1);
      reinterpret_cast<float4*>(&sK[r][0])[c4] = reinterpret_cast<const float4*>(k + ((size_t)jr * Hkv + hk) * D)[c4];
      reinterpret_cast<float4*>(&sV[r][0])[c4] = reinterpret_cast<const float4*>(v + ((size_t)jr * Hkv + hk) * D)[c4];
    }
    __syncthreads();
    for (int r = 0; r < kKeysStage; ++r) {
      if (j0 + r > row) break;                      // divergent exit is fine: no barrier inside
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) { s = fmaf(qr[c], sK[r][c], s); dp = fmaf(dor[c], sV[r][c], dp); }
      const float p = expf(s * scale - row_lse);
      const float ds = p * (dp - row_delta);
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(ds, sK[r][c], acc[c]);
    }
  }
  if (live) {
    float* out = dQ + ((size_t)row * Hq + h) * D;
#pragma unroll
    for (int c = 0; c < D; ++c) out[c] = acc[c] * scale;
  }
}

// dK/dV: block of 128 lanes owns 64 key rows of one KV head; lane pair (l, l^32) shares a key row
// and splits the head dimension.  Walks the scope's query runs at or after the tile, all heads
// of the group, in a fixed order.
template <int D>
__global__ __launch_bounds__(128) void dkdv_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                       const float* __restrict__ v, const float* __restrict__ dO,
                                                       const float* __restrict__ lse, const float* __restrict__ delta,
                                                       float* __restrict__ acc_dk, float* __restrict__ acc_dv,
                                                       float* __restrict__ dK, float* __restrict__ dV,
                                                       const KvItem* __restrict__ items, const Seg* __restrict__ segs, int T,
                                                       int Hq, int Hkv, float scale) {
  constexpr int HD = D / 2;
  __shared__ float sQ[kQStage][D];
  __shared__ float sDO[kQStage][D];
  __shared__ float sLse[kQStage], sDelta[kQStage];
  const KvItem it = items[blockIdx.x];
  const int hk = blockIdx.y, g = Hq / Hkv;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int key_local = wave * 32 + (lane % 32), half = lane / 32;
  const bool live = key_local < it.kv_rows;
  const int key = min(it.kv_row0 + key_local, T - 1);
  // an earlier unit's partial sum of this row is added (rows below load_until); rows no later unit reaches
  // (from final_from on) are written as dK/dV, the others into the accumulators
  const bool load_acc = key < it.load_until, store_final = key >= it.final_from;
  float kr[HD], vr[HD], dk[HD], dv[HD];
  const size_t kv_off = ((size_t)key * Hkv + hk) * D + half * HD;
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    kr[c] = k[kv_off + c];
    vr[c] = v[kv_off + c];
    dk[c] = (load_acc && live) ? acc_dk[kv_off + c] : 0.f;
    dv[c] = (load_acc && live) ? acc_dv[kv_off + c] : 0.f;
  }
  float dk_new[HD];                                   // scaled once at the end, like the definition
#pragma unroll
  for (int c = 0; c < HD; ++c) dk_new[c] = 0.f;
  for (int sgi = it.seg_begin; sgi < it.seg_end; ++sgi) {
    const Seg sg = segs[sgi];
    const int q_lo = max(sg.q_lo, it.kv_row0);
    for (int hh = 0; hh < g; ++hh) {
      const int h = hk * g + hh;
      for (int i0 = q_lo; i0 < sg.q_hi; i0 += kQStage) {
        __syncthreads();
        for (int e = tid; e < kQStage * (D / 4); e += 128) {
          const int r = e / (D / 4), c4 = e % (D / 4);
          const int ir = min(i0 + r, T - 1);
          reinterpret_cast<float4*>(&sQ[r][0])[c4] = reinterpret_cast<const float4*>(q + ((size_t)ir * Hq + h) * D)[c4];
          reinterpret_cast<float4*>(&sDO[r][0])[c4] = reinterpret_cast<const float4*>(dO + ((size_t)ir * Hq + h) * D)[c4];
        }
        if (tid < kQStage) {
          const int ir = min(i0 + tid, T - 1);
          sLse[tid] = lse[(size_t)h * T + ir];
          sDelta[tid] = delta[(size_t)h * T + ir];
        }
        __syncthreads();
        const int n_rows = min(kQStage, sg.q_hi - i0);
        for (int r = 0; r < n_rows; ++r) {
          float s = 0.f, dp = 0.f;
#pragma unroll
          for (int c = 0; c < HD; ++c) {
            s = fmaf(sQ[r][half * HD + c], kr[c], s);
            dp = fmaf(sDO[r][half * HD + c], vr[c], dp);
          }
          s += __shfl_xor(s, 32);
          dp += __shfl_xor(dp, 32);
          const float p = (i0 + r >= key) ? expf(s * scale - sLse[r]) : 0.f;
          const float ds = p * (dp - sDelta[r]);
#pragma unroll
          for (int c = 0; c < HD; ++c) {
            dv[c] = fmaf(p, sDO[r][half * HD + c], dv[c]);
            dk_new[c] = fmaf(ds, sQ[r][half * HD + c], dk_new[c]);
          }
        }
      }
    }
  }
  if (live) {
    float* out_k = store_final ? dK : acc_dk;
    float* out_v = store_final ? dV : acc_dv;
#pragma unroll
    for (int c = 0; c < HD; ++c) {
      out_k[kv_off + c] = dk[c] + dk_new[c] * scale;
      out_v[kv_off + c] = dv[c];
    }
  }
}

#define DISPATCH_D(D_, BODY)                 \
  switch (D_) {                              \
    case 16: { constexpr int D = 16; BODY; } break;   \
    case 32: { constexpr int D = 32; BODY; } break;   \
    case 64: { constexpr int D = 64; BODY; } break;   \
    case 128: { constexpr int D = 128; BODY; } break; \
    default: return (int)hipErrorInvalidValue;        \
  }

}  // namespace

int launch_fwd_f32(const LaunchCtx& c, const float* q, const float* k, const float* v, float* o, float* lse,
                   const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  DISPATCH_D(p.head_dim, hipLaunchKernelGGL(fwd_f32_kernel<D>, dim3(n_items, p.n_q_heads), dim3(kRowsF32), 0,
                                            (hipStream_t)c.stream, q, k, v, o, lse, items, (int)c.T, p.n_q_heads,
                                            p.n_kv_heads, p.scale));
  return (int)hipGetLastError();
}

int launch_bwd_delta_f32(const LaunchCtx& c, const float* o, const float* dO, float* delta, const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  DISPATCH_D(p.head_dim, hipLaunchKernelGGL(delta_f32_kernel<D>, dim3((unsigned)n_items), dim3(256), 0,
                                            (hipStream_t)c.stream, o, dO, delta, items, (int)c.T, p.n_q_heads));
  return (int)hipGetLastError();
}

int launch_bwd_dq_f32(const LaunchCtx& c, const float* q, const float* k, const float* v, const float* dO,
                      const float* lse, const float* delta, float* dQ, const QItem* items, int n_items) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  DISPATCH_D(p.head_dim, hipLaunchKernelGGL(dq_f32_kernel<D>, dim3(n_items, p.n_q_heads), dim3(kRowsF32), 0,
                                            (hipStream_t)c.stream, q, k, v, dO, lse, delta, dQ, items, (int)c.T,
                                            p.n_q_heads, p.n_kv_heads, p.scale));
  return (int)hipGetLastError();
}

int launch_bwd_dkdv_f32(const LaunchCtx& c, const float* q, const float* k, const float* v, const float* dO,
                        const float* lse, const float* delta, float* acc_dk, float* acc_dv, float* dK, float* dV,
                        const KvItem* items, int n_items, const Seg* segs) {
  if (n_items == 0) return 0;
  const slimattn_params& p = *c.p;
  DISPATCH_D(p.head_dim, hipLaunchKernelGGL(dkdv_f32_kernel<D>, dim3(n_items, p.n_kv_heads), dim3(128), 0,
                                            (hipStream_t)c.stream, q, k, v, dO, lse, delta, acc_dk, acc_dv, dK, dV, items,
                                            segs, (int)c.T, p.n_q_heads, p.n_kv_heads, p.scale));
  return (int)hipGetLastError();
}

}  // namespace slimattn
