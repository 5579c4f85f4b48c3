// Causal attention forward / backward, general path (any storage type, head_dim 64 or 128): one wave
// per query row (forward, dQ) or per key row (dK, dV), fp32 arithmetic, online softmax.  Used for the
// fp32 workload and as the fallback when the MFMA kernels do not apply.  q-head a reads kv-head
// a * n_kv / n_q; dK and dV are summed over the q-heads of a group.  Packed qkv rows:
// [q heads | k heads | v heads].  lse is [batch][n_q][seq], natural log.
#include "common.h"

namespace {

template <typename T, int DPL>   // DPL = head_dim / 64
__global__ __launch_bounds__(256) void attn_fwd_simple(const T* __restrict__ qkv, T* __restrict__ o,
                                                       float* __restrict__ lse, int seq, int n_q, int n_kv) {
  constexpr int D = 64 * DPL;
  __shared__ float qs[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t_raw = blockIdx.x * 4 + wave, a = blockIdx.y, b = blockIdx.z;
  const bool active = t_raw < seq;            // inactive waves redo the last row and skip the stores
  const int t = active ? t_raw : seq - 1;
  const int g = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const T* base = qkv + (size_t)b * seq * ld;
  const float scale = rsqrtf((float)D);
#pragma unroll
  for (int e = 0; e < DPL; ++e) qs[wave][lane + 64 * e] = to_f32(base[(size_t)t * ld + a * D + lane + 64 * e]) * scale;
  __syncthreads();
  const T* Kp = base + (size_t)(n_q + g) * D;
  const T* Vp = base + (size_t)(n_q + n_kv + g) * D;
  float m = -INFINITY, l = 0.f, acc[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
  for (int c0 = 0; c0 <= t; c0 += 64) {
    const int key = c0 + lane;
    const bool valid = key <= t;
    float s = -INFINITY;
    if (valid) {
      const T* kr = Kp + (size_t)key * ld;
      s = 0.f;
      for (int dd = 0; dd < D; ++dd) s = fmaf(qs[wave][dd], to_f32(kr[dd]), s);
    }
    const float mn = fmaxf(m, wave_max(s));
    const float p = valid ? expf(s - mn) : 0.f;
    const float alpha = expf(m - mn);
    l = l * alpha + wave_sum(p);
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[e] *= alpha;
    const int nj = min(64, t - c0 + 1);
    for (int j = 0; j < nj; ++j) {
      const float pj = __shfl(p, j, 64);
      const T* vr = Vp + (size_t)(c0 + j) * ld;
#pragma unroll
      for (int e = 0; e < DPL; ++e) acc[e] = fmaf(pj, to_f32(vr[lane + 64 * e]), acc[e]);
    }
    m = mn;
  }
  if (!active) return;
  T* orow = o + ((size_t)b * seq + t) * (n_q * D) + a * D;
#pragma unroll
  for (int e = 0; e < DPL; ++e) orow[lane + 64 * e] = from_f32<T>(acc[e] / l);
  if (lane == 0) lse[((size_t)b * n_q + a) * seq + t] = m + logf(l);
}

// per query row: D_t = <dO_t, O_t>, dQ_t = scale * sum_j dS_tj K_j
template <typename T, int DPL>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple(const T* __restrict__ qkv, const T* __restrict__ o,
                                                          const T* __restrict__ dout, const float* __restrict__ lse,
                                                          T* __restrict__ dqkv, float* __restrict__ Dws, int seq,
                                                          int n_q, int n_kv) {
  constexpr int D = 64 * DPL;
  __shared__ float qs[4][D];
  __shared__ float ds_[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t_raw = blockIdx.x * 4 + wave, a = blockIdx.y, b = blockIdx.z;
  const bool active = t_raw < seq;            // inactive waves redo the last row and skip the stores
  const int t = active ? t_raw : seq - 1;
  const int g = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const T* base = qkv + (size_t)b * seq * ld;
  const float scale = rsqrtf((float)D);
  const size_t orow = ((size_t)b * seq + t) * (n_q * D) + a * D;
  float dsum = 0.f;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    qs[wave][lane + 64 * e] = to_f32(base[(size_t)t * ld + a * D + lane + 64 * e]) * scale;
    float dv = to_f32(dout[orow + lane + 64 * e]);
    ds_[wave][lane + 64 * e] = dv;
    dsum += dv * to_f32(o[orow + lane + 64 * e]);
  }
  dsum = wave_sum(dsum);
  __syncthreads();
  const float L = lse[((size_t)b * n_q + a) * seq + t];
  if (lane == 0 && active) Dws[((size_t)b * n_q + a) * seq + t] = dsum;
  const T* Kp = base + (size_t)(n_q + g) * D;
  const T* Vp = base + (size_t)(n_q + n_kv + g) * D;
  float acc[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
  for (int c0 = 0; c0 <= t; c0 += 64) {
    const int key = c0 + lane;
    float dS = 0.f;
    if (key <= t) {
      const T* kr = Kp + (size_t)key * ld;
      const T* vr = Vp + (size_t)key * ld;
      float s = 0.f, dp = 0.f;
      for (int dd = 0; dd < D; ++dd) {
        s = fmaf(qs[wave][dd], to_f32(kr[dd]), s);
        dp = fmaf(ds_[wave][dd], to_f32(vr[dd]), dp);
      }
      dS = expf(s - L) * (dp - dsum);
    }
    const int nj = min(64, t - c0 + 1);
    for (int j = 0; j < nj; ++j) {
      const float dj = __shfl(dS, j, 64);
      const T* kr = Kp + (size_t)(c0 + j) * ld;
#pragma unroll
      for (int e = 0; e < DPL; ++e) acc[e] = fmaf(dj, to_f32(kr[lane + 64 * e]), acc[e]);
    }
  }
  if (!active) return;
  T* dq = dqkv + ((size_t)b * seq + t) * ld + a * D;
#pragma unroll
  for (int e = 0; e < DPL; ++e) dq[lane + 64 * e] = from_f32<T>(acc[e] * scale);
}

// per key row and kv head: dV = sum_t P_t dO_t, dK = scale * sum_t dS_t Q_t over the group's q heads
template <typename T, int DPL>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ Dws,
                                                           T* __restrict__ dqkv, int seq, int n_q, int n_kv) {
  constexpr int D = 64 * DPL;
  __shared__ float ks[4][D];
  __shared__ float vs[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tk_raw = blockIdx.x * 4 + wave, g = blockIdx.y, b = blockIdx.z;
  const bool active = tk_raw < seq;
  const int tk = active ? tk_raw : seq - 1;
  const int ld = (n_q + 2 * n_kv) * D;
  const T* base = qkv + (size_t)b * seq * ld;
  const float scale = rsqrtf((float)D);
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    ks[wave][lane + 64 * e] = to_f32(base[(size_t)tk * ld + (n_q + g) * D + lane + 64 * e]) * scale;
    vs[wave][lane + 64 * e] = to_f32(base[(size_t)tk * ld + (n_q + n_kv + g) * D + lane + 64 * e]);
  }
  __syncthreads();
  float dk[DPL], dv[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) { dk[e] = 0.f; dv[e] = 0.f; }
  const int rep = n_q / n_kv;
  for (int a = g * rep; a < (g + 1) * rep; ++a) {
    const float* Lp = lse + ((size_t)b * n_q + a) * seq;
    const float* Dp = Dws + ((size_t)b * n_q + a) * seq;
    for (int c0 = (tk / 64) * 64; c0 < seq; c0 += 64) {
      const int tq = c0 + lane;
      float p = 0.f, dS = 0.f;
      if (tq >= tk && tq < seq) {
        const T* qr = base + (size_t)tq * ld + a * D;
        const T* dor = dout + ((size_t)b * seq + tq) * (n_q * D) + a * D;
        float s = 0.f, dp = 0.f;
        for (int dd = 0; dd < D; ++dd) {
          s = fmaf(ks[wave][dd], to_f32(qr[dd]), s);
          dp = fmaf(vs[wave][dd], to_f32(dor[dd]), dp);
        }
        p = expf(s - Lp[tq]);
        dS = p * (dp - Dp[tq]);
      }
      const int j0 = max(0, tk - c0), j1 = min(64, seq - c0);
      for (int j = j0; j < j1; ++j) {
        const float pj = __shfl(p, j, 64), dj = __shfl(dS, j, 64);
        const T* qr = base + (size_t)(c0 + j) * ld + a * D;
        const T* dor = dout + ((size_t)b * seq + c0 + j) * (n_q * D) + a * D;
#pragma unroll
        for (int e = 0; e < DPL; ++e) {
          dv[e] = fmaf(pj, to_f32(dor[lane + 64 * e]), dv[e]);
          dk[e] = fmaf(dj, to_f32(qr[lane + 64 * e]), dk[e]);
        }
      }
    }
  }
  if (!active) return;
  T* dkr = dqkv + ((size_t)b * seq + tk) * ld + (n_q + g) * D;
  T* dvr = dqkv + ((size_t)b * seq + tk) * ld + (n_q + n_kv + g) * D;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    dkr[lane + 64 * e] = from_f32<T>(dk[e] * scale);
    dvr[lane + 64 * e] = from_f32<T>(dv[e]);
  }
}

template <typename T, int DPL>
hipError_t fwd_t(const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv, hipStream_t s) {
  hipLaunchKernelGGL((attn_fwd_simple<T, DPL>), dim3((seq + 3) / 4, n_q, batch), dim3(256), 0, s, (const T*)qkv, (T*)o, lse, seq, n_q, n_kv);
  return hipGetLastError();
}
template <typename T, int DPL>
hipError_t bwd_t(const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv, float* ws, int seq,
                 int batch, int n_q, int n_kv, hipStream_t s) {
  hipLaunchKernelGGL((attn_bwd_dq_simple<T, DPL>), dim3((seq + 3) / 4, n_q, batch), dim3(256), 0, s, (const T*)qkv,
      (const T*)o, (const T*)dout, lse, (T*)dqkv, ws, seq, n_q, n_kv);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkv_simple<T, DPL>), dim3((seq + 3) / 4, n_kv, batch), dim3(256), 0, s, (const T*)qkv,
      (const T*)dout, lse, ws, (T*)dqkv, seq, n_q, n_kv);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd_simple(int dtype, const void* qkv, void* o, float* lse, int seq, int batch, int n_q,
                                  int n_kv, int d, hipStream_t s) {
  if (dtype == DT_BF16) {
    if (d == 64) return fwd_t<bf16_t, 1>(qkv, o, lse, seq, batch, n_q, n_kv, s);
    if (d == 128) return fwd_t<bf16_t, 2>(qkv, o, lse, seq, batch, n_q, n_kv, s);
  } else {
    if (d == 64) return fwd_t<float, 1>(qkv, o, lse, seq, batch, n_q, n_kv, s);
    if (d == 128) return fwd_t<float, 2>(qkv, o, lse, seq, batch, n_q, n_kv, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_bwd_simple(int dtype, const void* qkv, const void* o, const void* dout, const float* lse,
                                  void* dqkv, float* ws, int seq, int batch, int n_q, int n_kv, int d, hipStream_t s) {
  if (dtype == DT_BF16) {
    if (d == 64) return bwd_t<bf16_t, 1>(qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, s);
    if (d == 128) return bwd_t<bf16_t, 2>(qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, s);
  } else {
    if (d == 64) return bwd_t<float, 1>(qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, s);
    if (d == 128) return bwd_t<float, 2>(qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, s);
  }
  return hipErrorInvalidValue;
}
