// HBM-bound fused elementwise kernels of a stage: the non-linear parts that the paper's stage model
// folds into sigma(.) (Sec. 2.2) — RMSNorm / LayerNorm, SwiGLU / GELU, rotary — forward and backward,
// plus helpers (weight transpose, rotary table, buffer checksum).  All arithmetic is fp32 on 16-byte
// vector accesses of the storage type; rows are tokens.
#include "common.h"

namespace {

constexpr int NT = 256;
constexpr int MAXC = 4;   // 16-byte chunks per thread per row: hidden <= 256 * 4 * (4 | 8)

__device__ __forceinline__ float block_sum(float v, float* red /* [2][4] */, int parity) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[parity * 4 + wave] = v;
  __syncthreads();
  return red[parity * 4] + red[parity * 4 + 1] + red[parity * 4 + 2] + red[parity * 4 + 3];
}

// ---- norm forward: one row per workgroup ------------------------------------------------------------
template <typename T, bool LN>
__global__ __launch_bounds__(NT) void norm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                      const T* __restrict__ beta, T* __restrict__ out,
                                                      float* __restrict__ stats, int rows, int h, float eps) {
  typedef Vec16<T> V;
  __shared__ float red[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int nvec = h / V::N;
  V xv[MAXC];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int ci = tid + c * NT;
    if (ci < nvec) {
      xv[c] = *reinterpret_cast<const V*>(x + (size_t)row * h + ci * V::N);
#pragma unroll
      for (int e = 0; e < V::N; ++e) { float f = xv[c].get(e); s1 += f; s2 += f * f; }
    }
  }
  float mean = 0.f;
  if (LN) {
    mean = block_sum(s1, red, 0) / h;
    // two-pass variance for accuracy
    s2 = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = tid + c * NT;
      if (ci < nvec)
#pragma unroll
        for (int e = 0; e < V::N; ++e) { float f = xv[c].get(e) - mean; s2 += f * f; }
    }
  }
  const float var = block_sum(s2, red, 1) / h;
  const float r = rsqrtf(var + eps);
  if (tid == 0) {
    if (LN) { stats[2 * row] = mean; stats[2 * row + 1] = r; } else stats[row] = r;
  }
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int ci = tid + c * NT;
    if (ci < nvec) {
      V g = *reinterpret_cast<const V*>(gamma + ci * V::N), o;
      V b;
      if (LN) b = *reinterpret_cast<const V*>(beta + ci * V::N);
#pragma unroll
      for (int e = 0; e < V::N; ++e) {
        float f = (xv[c].get(e) - mean) * r * g.get(e);
        if (LN) f += b.get(e);
        o.set(e, f);
      }
      *reinterpret_cast<V*>(out + (size_t)row * h + ci * V::N) = o;
    }
  }
}

// ---- norm backward: workgroup b handles rows b, b + gridDim.x, ...; per-column partial sums of the
// gain / bias gradients stay in registers and are written once per workgroup -------------------------
template <typename T, bool LN>
__global__ __launch_bounds__(NT) void norm_bwd_kernel(const T* __restrict__ dn, const T* __restrict__ x,
                                                      const float* __restrict__ stats, const T* __restrict__ gamma,
                                                      const T* __restrict__ dres, T* __restrict__ dx,
                                                      float* __restrict__ partial, int rows, int h) {
  typedef Vec16<T> V;
  __shared__ float red[16];
  const int tid = threadIdx.x;
  const int nvec = h / V::N;
  float pg[MAXC][V::N], pb[MAXC][V::N];
  V gv[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int ci = tid + c * NT;
    if (ci < nvec) gv[c] = *reinterpret_cast<const V*>(gamma + ci * V::N);
#pragma unroll
    for (int e = 0; e < V::N; ++e) { pg[c][e] = 0.f; pb[c][e] = 0.f; }
  }
  // three register sets: the loads of the next two rows are in flight while the current one is reduced and
  // written (with one workgroup per compute unit the bytes in flight, not the arithmetic, set the pace)
  V xv[3][MAXC], dv[3][MAXC], rv[3][MAXC];
  float mean_[3], r_[3];
  auto load_row = [&](int buf, int row) {
    if (LN) { mean_[buf] = stats[2 * row]; r_[buf] = stats[2 * row + 1]; } else { mean_[buf] = 0.f; r_[buf] = stats[row]; }
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = tid + c * NT;
      if (ci < nvec) {
        xv[buf][c] = *reinterpret_cast<const V*>(x + (size_t)row * h + ci * V::N);
        dv[buf][c] = *reinterpret_cast<const V*>(dn + (size_t)row * h + ci * V::N);
        if (dres) rv[buf][c] = *reinterpret_cast<const V*>(dres + (size_t)row * h + ci * V::N);
      }
    }
  };
  int it = 0;
  auto process = [&](int buf, int row) {
    const float mean = mean_[buf], r = r_[buf];
    float sg = 0.f, sgx = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = tid + c * NT;
      if (ci < nvec) {
#pragma unroll
        for (int e = 0; e < V::N; ++e) {
          float xh = (xv[buf][c].get(e) - mean) * r;
          float d = dv[buf][c].get(e);
          float g = d * gv[c].get(e);
          sg += g;
          sgx += g * xh;
          pg[c][e] += d * xh;
          pb[c][e] += d;
        }
      }
    }
    const int par = (it & 1) * 2;
    ++it;
    // two reductions share one barrier: pack both partials before the sync
    sgx = wave_sum(sgx);
    sg = wave_sum(sg);
    const int wave = tid >> 6;
    if ((tid & 63) == 0) { red[par * 4 + wave] = sgx; red[(par + 1) * 4 + wave] = sg; }
    __syncthreads();
    const float mgx = (red[par * 4] + red[par * 4 + 1] + red[par * 4 + 2] + red[par * 4 + 3]) / h;
    const float mg = LN ? (red[(par + 1) * 4] + red[(par + 1) * 4 + 1] + red[(par + 1) * 4 + 2] + red[(par + 1) * 4 + 3]) / h : 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = tid + c * NT;
      if (ci < nvec) {
        V o;
#pragma unroll
        for (int e = 0; e < V::N; ++e) {
          float xh = (xv[buf][c].get(e) - mean) * r;
          float g = dv[buf][c].get(e) * gv[c].get(e);
          float d = r * (g - mg - xh * mgx);
          if (dres) d += rv[buf][c].get(e);
          o.set(e, d);
        }
        *reinterpret_cast<V*>(dx + (size_t)row * h + ci * V::N) = o;
      }
    }
  };
  const int gd = gridDim.x;
  int row = blockIdx.x;
  if (row < rows) load_row(0, row);
  if (row + gd < rows) load_row(1, row + gd);
  for (; row < rows; row += 3 * gd) {
    const int r1 = row + gd, r2 = row + 2 * gd, r3 = row + 3 * gd, r4 = row + 4 * gd;
    if (r2 < rows) load_row(2, r2);
    process(0, row);
    if (r1 < rows) {
      if (r3 < rows) load_row(0, r3);
      process(1, r1);
    }
    if (r2 < rows) {
      if (r4 < rows) load_row(1, r4);
      process(2, r2);
    }
  }
  float* pgo = partial + (size_t)blockIdx.x * h;
  float* pbo = partial + (size_t)(gridDim.x + blockIdx.x) * h;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int ci = tid + c * NT;
    if (ci < nvec)
#pragma unroll
      for (int e = 0; e < V::N; ++e) {
        pgo[ci * V::N + e] = pg[c][e];
        if (LN) pbo[ci * V::N + e] = pb[c][e];
      }
  }
}

// Narrow rows (at most 64 * MAXC 16-byte chunks): one row per WAVE, so the two row sums need no barrier and a
// workgroup has four rows in flight; the four waves' column partials are added through LDS at the end, in wave
// order, into the workgroup's one row of partial sums.
template <typename T, bool LN>
__global__ __launch_bounds__(NT) void norm_bwd_wave_kernel(const T* __restrict__ dn, const T* __restrict__ x,
                                                           const float* __restrict__ stats, const T* __restrict__ gamma,
                                                           const T* __restrict__ dres, T* __restrict__ dx,
                                                           float* __restrict__ partial, int rows, int h) {
  typedef Vec16<T> V;
  constexpr int MAXH = 64 * MAXC * V::N;
  __shared__ float comb[4 * MAXH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nvec = h / V::N;
  float pg[MAXC][V::N], pb[MAXC][V::N];
  V gv[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int ci = lane + c * 64;
    if (ci < nvec) gv[c] = *reinterpret_cast<const V*>(gamma + ci * V::N);
#pragma unroll
    for (int e = 0; e < V::N; ++e) { pg[c][e] = 0.f; pb[c][e] = 0.f; }
  }
  V xv[2][MAXC], dv[2][MAXC], rv[2][MAXC];
  float mean_[2], r_[2];
  auto load_row = [&](int buf, int row) {
    if (LN) { mean_[buf] = stats[2 * row]; r_[buf] = stats[2 * row + 1]; } else { mean_[buf] = 0.f; r_[buf] = stats[row]; }
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = lane + c * 64;
      if (ci < nvec) {
        xv[buf][c] = *reinterpret_cast<const V*>(x + (size_t)row * h + ci * V::N);
        dv[buf][c] = *reinterpret_cast<const V*>(dn + (size_t)row * h + ci * V::N);
        if (dres) rv[buf][c] = *reinterpret_cast<const V*>(dres + (size_t)row * h + ci * V::N);
      }
    }
  };
  auto process = [&](int buf, int row) {
    const float mean = mean_[buf], r = r_[buf];
    float sg = 0.f, sgx = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = lane + c * 64;
      if (ci < nvec) {
#pragma unroll
        for (int e = 0; e < V::N; ++e) {
          float xh = (xv[buf][c].get(e) - mean) * r;
          float d = dv[buf][c].get(e);
          float g = d * gv[c].get(e);
          sg += g;
          sgx += g * xh;
          pg[c][e] += d * xh;
          pb[c][e] += d;
        }
      }
    }
    const float mgx = wave_sum(sgx) / h;
    const float mg = LN ? wave_sum(sg) / h : 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = lane + c * 64;
      if (ci < nvec) {
        V o;
#pragma unroll
        for (int e = 0; e < V::N; ++e) {
          float xh = (xv[buf][c].get(e) - mean) * r;
          float g = dv[buf][c].get(e) * gv[c].get(e);
          float d = r * (g - mg - xh * mgx);
          if (dres) d += rv[buf][c].get(e);
          o.set(e, d);
        }
        *reinterpret_cast<V*>(dx + (size_t)row * h + ci * V::N) = o;
      }
    }
  };
  const int gd = gridDim.x * 4;
  int row = blockIdx.x * 4 + wave;
  if (row < rows) load_row(0, row);
  for (; row < rows; row += 2 * gd) {
    const int r1 = row + gd, r2 = row + 2 * gd;
    if (r1 < rows) load_row(1, r1);
    process(0, row);
    if (r1 < rows) {
      if (r2 < rows) load_row(0, r2);
      process(1, r1);
    }
  }
  for (int pass = 0; pass < (LN ? 2 : 1); ++pass) {
    if (pass) __syncthreads();
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      int ci = lane + c * 64;
      if (ci < nvec)
#pragma unroll
        for (int e = 0; e < V::N; ++e) comb[wave * MAXH + ci * V::N + e] = pass ? pb[c][e] : pg[c][e];
    }
    __syncthreads();
    float* out = partial + (size_t)(pass * gridDim.x + blockIdx.x) * h;
    for (int col = tid; col < h; col += NT)
      out[col] = ((comb[col] + comb[MAXH + col]) + comb[2 * MAXH + col]) + comb[3 * MAXH + col];
  }
}

// sums the per-workgroup partials column-wise and adds them into the caller's fp32 accumulators (overwrite: stores
// them instead): workgroup = 32 columns x 8 row groups, fixed summation order (deterministic)
__global__ __launch_bounds__(256) void norm_bwd_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dgamma,
                                                              float* __restrict__ dbeta, int nb, int h, int overwrite) {
  __shared__ float red[8][33];
  const int cx = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + cx;
  const float* p = partial + (size_t)blockIdx.y * nb * h;
  // four independent partial sums keep four loads in flight per lane; fixed combination order
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (col < h) {
    int b = rg;
    for (; b + 24 < nb; b += 32) {
      s0 += p[(size_t)b * h + col];
      s1 += p[(size_t)(b + 8) * h + col];
      s2 += p[(size_t)(b + 16) * h + col];
      s3 += p[(size_t)(b + 24) * h + col];
    }
    for (; b < nb; b += 8) s0 += p[(size_t)b * h + col];
  }
  red[rg][cx] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (rg == 0 && col < h) {
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) t += red[r][cx];
    float* dst = blockIdx.y == 0 ? dgamma : dbeta;
    dst[col] = overwrite ? t : dst[col] + t;
  }
}

// ---- MLP activations --------------------------------------------------------------------------------
__device__ __forceinline__ float sigmoidf_(float x) { return 1.f / (1.f + expf(-x)); }

template <typename T, bool SWIGLU>
__global__ void act_fwd_kernel(const T* __restrict__ gu, T* __restrict__ a, int rows, int f) {
  typedef Vec16<T> V;
  const int nvec = f / V::N;
  const size_t total = (size_t)rows * nvec;
  const int ldg = SWIGLU ? 2 * f : f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    int row = i / nvec, c = i % nvec;
    V g = *reinterpret_cast<const V*>(gu + (size_t)row * ldg + c * V::N), u, o;
    if (SWIGLU) u = *reinterpret_cast<const V*>(gu + (size_t)row * ldg + f + c * V::N);
#pragma unroll
    for (int e = 0; e < V::N; ++e) {
      float x = g.get(e);
      if (SWIGLU) o.set(e, x * sigmoidf_(x) * u.get(e));
      else o.set(e, 0.5f * x * (1.f + erff(x * 0.70710678118654752f)));
    }
    *reinterpret_cast<V*>(a + (size_t)row * f + c * V::N) = o;
  }
}

// dgu may alias gu (each thread reads its elements before writing the same positions)
template <typename T, bool SWIGLU>
__global__ void act_bwd_kernel(const T* __restrict__ da, const T* gu, T* dgu, int rows, int f) {
  typedef Vec16<T> V;
  const int nvec = f / V::N;
  const size_t total = (size_t)rows * nvec;
  const int ldg = SWIGLU ? 2 * f : f;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    int row = i / nvec, c = i % nvec;
    V d = *reinterpret_cast<const V*>(da + (size_t)row * f + c * V::N);
    V g = *reinterpret_cast<const V*>(gu + (size_t)row * ldg + c * V::N), u, og, ou;
    if (SWIGLU) u = *reinterpret_cast<const V*>(gu + (size_t)row * ldg + f + c * V::N);
#pragma unroll
    for (int e = 0; e < V::N; ++e) {
      float x = g.get(e), dd = d.get(e);
      if (SWIGLU) {
        float s = sigmoidf_(x);
        og.set(e, dd * u.get(e) * s * (1.f + x * (1.f - s)));
        ou.set(e, dd * x * s);
      } else {
        float Phi = 0.5f * (1.f + erff(x * 0.70710678118654752f));
        float phi = 0.39894228040143268f * expf(-0.5f * x * x);
        og.set(e, dd * (Phi + x * phi));
      }
    }
    *reinterpret_cast<V*>(dgu + (size_t)row * ldg + c * V::N) = og;
    if (SWIGLU) *reinterpret_cast<V*>(dgu + (size_t)row * ldg + f + c * V::N) = ou;
  }
}

// ---- rotary -----------------------------------------------------------------------------------------
// table[pos][k] = (cos, sin)(pos * base^(-2k/d)), k < d/2, evaluated in fp64 once
__global__ void rope_table_kernel(float2* __restrict__ table, int seq, int half, double base) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= seq * half) return;
  int pos = i / half, k = i % half;
  double theta = pow(base, -(double)k / (double)half);
  double ang = (double)pos * theta;
  table[i] = make_float2((float)cos(ang), (float)sin(ang));
}

// rotates the q and k heads of packed qkv rows, pairing element k with k + d/2; sign = -1 applies the
// transposed rotation (gradients).  When dst != src the v part is copied as well.
template <typename T, int HG>
__global__ void rope_kernel(const T* src, T* dst, const float2* __restrict__ table, int rows, int seq, int n_rot,
                            int n_v, int d, float sign, int do_rotate) {
  typedef Vec16<T> V;
  const int half = d / 2, vph = half / V::N;        // vectors per half head
  const int ld = (n_rot + n_v) * d;
  const int groups = n_rot / HG;                    // HG heads share the cos / sin values a thread has fetched
  const size_t rot_items = (size_t)rows * groups * vph;
  const size_t cp_items = (src != dst) ? (size_t)rows * n_v * (d / V::N) : 0;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < rot_items + cp_items; i += (size_t)gridDim.x * blockDim.x) {
    if (i < rot_items) {
      int c = i % vph;
      size_t t = i / vph;
      int grp = t % groups, row = t / groups;
      int pos = row % seq;
      float cs[V::N], sn[V::N];
#pragma unroll
      for (int e = 0; e < V::N; ++e) {
        cs[e] = 1.f; sn[e] = 0.f;
        if (do_rotate) { float2 cssn = table[(size_t)pos * half + c * V::N + e]; cs[e] = cssn.x; sn[e] = sign * cssn.y; }
      }
      V lo[HG], hi[HG];
#pragma unroll
      for (int g = 0; g < HG; ++g) {
        const size_t off = (size_t)row * ld + (size_t)(grp * HG + g) * d + c * V::N;
        lo[g] = *reinterpret_cast<const V*>(src + off);
        hi[g] = *reinterpret_cast<const V*>(src + off + half);
      }
#pragma unroll
      for (int g = 0; g < HG; ++g) {
        const size_t off = (size_t)row * ld + (size_t)(grp * HG + g) * d + c * V::N;
        V olo, ohi;
#pragma unroll
        for (int e = 0; e < V::N; ++e) {
          float a = lo[g].get(e), b = hi[g].get(e);
          olo.set(e, a * cs[e] - b * sn[e]);
          ohi.set(e, b * cs[e] + a * sn[e]);
        }
        *reinterpret_cast<V*>(dst + off) = olo;
        *reinterpret_cast<V*>(dst + off + half) = ohi;
      }
    } else {
      size_t k = i - rot_items;
      int per_row = n_v * (d / V::N);
      int row = k / per_row, c = k % per_row;
      size_t off = (size_t)row * ld + (size_t)n_rot * d + c * V::N;
      *reinterpret_cast<V*>(dst + off) = *reinterpret_cast<const V*>(src + off);
    }
  }
}

// ---- weights into slabs (once per weight update): the GEMM's B operand B[n][k], n < N, k < K (K % 64 == 0), stored
// so that the 256 rows x 64 columns a workgroup loads per k-tile are consecutive in memory: slab (n / 256, k / 64) at
// element offset ((n / 256) * (K / 64) + k / 64) * 16384, row-major inside, rows past N zero.
// TRANSPOSED = false: B[n][k] = src[n * K + k]; true: B[n][k] = src[k * N + n] (the transposed weight)
// pair_f > 0 (not TRANSPOSED): the source is a [gate | up] weight with pair_f rows each; the 64 slab rows of this
// workgroup (tile t = n0 / 256, wave half w, q = 0 gate / 1 up) come from source rows q pair_f + 128 t + 64 w + 0..63
template <bool TRANSPOSED>
__global__ void slab_kernel(const unsigned short* __restrict__ src, unsigned short* __restrict__ dst, int N, int K, int pair_f) {
  __shared__ unsigned short tile[64][65];
  const int n0 = blockIdx.y * 64, k0 = blockIdx.x * 64;
  const int s0 = pair_f > 0 ? ((n0 >> 6) & 1) * pair_f + (n0 >> 8) * 128 + ((n0 >> 7) & 1) * 64 : n0;   // first source row
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    const int hi = e / 64, lo = e % 64;               // lo runs along the source's contiguous direction
    const int nn = TRANSPOSED ? lo : hi, kk = TRANSPOSED ? hi : lo;
    unsigned short v = 0;
    if (n0 + nn < N) v = TRANSPOSED ? src[(size_t)(k0 + kk) * N + n0 + nn] : src[(size_t)(s0 + nn) * K + k0 + kk];
    tile[nn][kk] = v;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    const int nn = e / 64, kk = e % 64, n = n0 + nn;
    dst[((size_t)(n / 256) * (K / 64) + k0 / 64) * 16384 + (size_t)(n % 256) * 64 + kk] = tile[nn][kk];
  }
}

// ---- transpose (weights, once per weight update) ------------------------------------------------------
template <typename T>
__global__ void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows, int cols) {
  __shared__ T tile[64][65];
  int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    int r = e / 64, c = e % 64;
    if (r0 + r < rows && c0 + c < cols) tile[r][c] = src[(size_t)(r0 + r) * cols + c0 + c];
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += blockDim.x) {
    int c = e / 64, r = e % 64;
    if (r0 + r < rows && c0 + c < cols) dst[(size_t)(c0 + c) * rows + r0 + r] = tile[r][c];
  }
}

// ---- checksum: out[0] = sum of 64-bit words (mod 2^64), out[1] = xor of 64-bit words ---------------------
__global__ void checksum_zero_kernel(unsigned long long* out) { out[0] = 0ull; out[1] = 0ull; }
__global__ void checksum_kernel(const unsigned long long* __restrict__ w, size_t n, unsigned long long* out) {
  unsigned long long s = 0, x = 0;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    unsigned long long v = w[i];
    s += v;
    x ^= v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    s += __shfl_xor(s, o, 64);
    x ^= __shfl_xor(x, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(&out[0], s);
    atomicXor(&out[1], x);
  }
}

int grid_for(size_t items, int block) {
  size_t g = (items + block - 1) / block;
  return (int)(g < 1 ? 1 : (g > 256 * 32 ? 256 * 32 : g));
}

template <typename T> bool norm_shape_ok(int h) { return h > 0 && h % Vec16<T>::N == 0 && h / Vec16<T>::N <= NT * MAXC; }

}  // namespace

hipError_t launch_norm_fwd(int dtype, int family, const void* x, const void* gamma, const void* beta, void* out,
                           float* stats, int rows, int h, float eps, hipStream_t s) {
  if (rows <= 0) return hipErrorInvalidValue;
  const bool ln = family == FAM_GPT;
  if (dtype == DT_BF16) {
    if (!norm_shape_ok<bf16_t>(h)) return hipErrorInvalidValue;
    if (ln) hipLaunchKernelGGL((norm_fwd_kernel<bf16_t, true>), dim3(rows), dim3(NT), 0, s, (const bf16_t*)x,
        (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)out, stats, rows, h, eps);
    else hipLaunchKernelGGL((norm_fwd_kernel<bf16_t, false>), dim3(rows), dim3(NT), 0, s, (const bf16_t*)x,
        (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)out, stats, rows, h, eps);
  } else {
    if (!norm_shape_ok<float>(h)) return hipErrorInvalidValue;
    if (ln) hipLaunchKernelGGL((norm_fwd_kernel<float, true>), dim3(rows), dim3(NT), 0, s, (const float*)x,
        (const float*)gamma, (const float*)beta, (float*)out, stats, rows, h, eps);
    else hipLaunchKernelGGL((norm_fwd_kernel<float, false>), dim3(rows), dim3(NT), 0, s, (const float*)x,
        (const float*)gamma, (const float*)beta, (float*)out, stats, rows, h, eps);
  }
  return hipGetLastError();
}

// Workgroups of the norm backward kernels = rows of per-workgroup gain / bias partials: one per compute unit of the
// 256-unit part.  512 cost 9-17 % more (twice the partials to write and to reduce), counts that do not divide the
// units evenly 20-60 % more.
int norm_bwd_partial_rows(int rows) { return rows < 256 ? rows : 256; }

hipError_t launch_norm_bwd(int dtype, int family, const void* dn, const void* x, const float* stats,
                           const void* gamma, const void* dres, void* dx, float* partial, float* dgamma,
                           float* dbeta, int rows, int h, hipStream_t s, int overwrite) {
  if (rows <= 0) return hipErrorInvalidValue;
  const bool ln = family == FAM_GPT;
  const int nb = norm_bwd_partial_rows(rows);
  if (dtype == DT_BF16) {
    if (!norm_shape_ok<bf16_t>(h)) return hipErrorInvalidValue;
    const bool narrow = h / 8 <= 64 * MAXC && rows >= 4 * nb;   // one row per wave
    if (ln && narrow) hipLaunchKernelGGL((norm_bwd_wave_kernel<bf16_t, true>), dim3(nb), dim3(NT), 0, s, (const bf16_t*)dn,
        (const bf16_t*)x, stats, (const bf16_t*)gamma, (const bf16_t*)dres, (bf16_t*)dx, partial, rows, h);
    else if (narrow) hipLaunchKernelGGL((norm_bwd_wave_kernel<bf16_t, false>), dim3(nb), dim3(NT), 0, s, (const bf16_t*)dn,
        (const bf16_t*)x, stats, (const bf16_t*)gamma, (const bf16_t*)dres, (bf16_t*)dx, partial, rows, h);
    else if (ln) hipLaunchKernelGGL((norm_bwd_kernel<bf16_t, true>), dim3(nb), dim3(NT), 0, s, (const bf16_t*)dn,
        (const bf16_t*)x, stats, (const bf16_t*)gamma, (const bf16_t*)dres, (bf16_t*)dx, partial, rows, h);
    else hipLaunchKernelGGL((norm_bwd_kernel<bf16_t, false>), dim3(nb), dim3(NT), 0, s, (const bf16_t*)dn, (const bf16_t*)x,
        stats, (const bf16_t*)gamma, (const bf16_t*)dres, (bf16_t*)dx, partial, rows, h);
  } else {
    if (!norm_shape_ok<float>(h)) return hipErrorInvalidValue;
    const bool narrow = h / 4 <= 64 * MAXC && rows >= 4 * nb;
    if (ln && narrow) hipLaunchKernelGGL((norm_bwd_wave_kernel<float, true>), dim3(nb), dim3(NT), 0, s, (const float*)dn,
        (const float*)x, stats, (const float*)gamma, (const float*)dres, (float*)dx, partial, rows, h);
    else if (narrow) hipLaunchKernelGGL((norm_bwd_wave_kernel<float, false>), dim3(nb), dim3(NT), 0, s, (const float*)dn,
        (const float*)x, stats, (const float*)gamma, (const float*)dres, (float*)dx, partial, rows, h);
    else if (ln) hipLaunchKernelGGL((norm_bwd_kernel<float, true>), dim3(nb), dim3(NT), 0, s, (const float*)dn,
        (const float*)x, stats, (const float*)gamma, (const float*)dres, (float*)dx, partial, rows, h);
    else hipLaunchKernelGGL((norm_bwd_kernel<float, false>), dim3(nb), dim3(NT), 0, s, (const float*)dn, (const float*)x,
        stats, (const float*)gamma, (const float*)dres, (float*)dx, partial, rows, h);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(norm_bwd_reduce_kernel, dim3((h + 31) / 32, ln ? 2 : 1), dim3(256), 0, s, partial, dgamma, dbeta, nb, h, overwrite);
  return hipGetLastError();
}

hipError_t launch_act_fwd(int dtype, int family, const void* gu, void* a, int rows, int f, hipStream_t s) {
  if (rows <= 0 || f <= 0) return hipErrorInvalidValue;
  const bool sw = family == FAM_LLAMA;
  if (dtype == DT_BF16) {
    if (f % 8) return hipErrorInvalidValue;
    int g = grid_for((size_t)rows * (f / 8), 256);
    if (sw) hipLaunchKernelGGL((act_fwd_kernel<bf16_t, true>), dim3(g), dim3(256), 0, s, (const bf16_t*)gu, (bf16_t*)a, rows, f);
    else hipLaunchKernelGGL((act_fwd_kernel<bf16_t, false>), dim3(g), dim3(256), 0, s, (const bf16_t*)gu, (bf16_t*)a, rows, f);
  } else {
    if (f % 4) return hipErrorInvalidValue;
    int g = grid_for((size_t)rows * (f / 4), 256);
    if (sw) hipLaunchKernelGGL((act_fwd_kernel<float, true>), dim3(g), dim3(256), 0, s, (const float*)gu, (float*)a, rows, f);
    else hipLaunchKernelGGL((act_fwd_kernel<float, false>), dim3(g), dim3(256), 0, s, (const float*)gu, (float*)a, rows, f);
  }
  return hipGetLastError();
}

hipError_t launch_act_bwd(int dtype, int family, const void* da, const void* gu, void* dgu, int rows, int f,
                          hipStream_t s) {
  if (rows <= 0 || f <= 0) return hipErrorInvalidValue;
  const bool sw = family == FAM_LLAMA;
  if (dtype == DT_BF16) {
    if (f % 8) return hipErrorInvalidValue;
    int g = grid_for((size_t)rows * (f / 8), 256);
    if (sw) hipLaunchKernelGGL((act_bwd_kernel<bf16_t, true>), dim3(g), dim3(256), 0, s, (const bf16_t*)da, (const bf16_t*)gu, (bf16_t*)dgu, rows, f);
    else hipLaunchKernelGGL((act_bwd_kernel<bf16_t, false>), dim3(g), dim3(256), 0, s, (const bf16_t*)da, (const bf16_t*)gu, (bf16_t*)dgu, rows, f);
  } else {
    if (f % 4) return hipErrorInvalidValue;
    int g = grid_for((size_t)rows * (f / 4), 256);
    if (sw) hipLaunchKernelGGL((act_bwd_kernel<float, true>), dim3(g), dim3(256), 0, s, (const float*)da, (const float*)gu, (float*)dgu, rows, f);
    else hipLaunchKernelGGL((act_bwd_kernel<float, false>), dim3(g), dim3(256), 0, s, (const float*)da, (const float*)gu, (float*)dgu, rows, f);
  }
  return hipGetLastError();
}

hipError_t launch_rope_table(float* table, int seq, int d, float base, hipStream_t s) {
  if (seq <= 0 || d <= 0 || (d & 1)) return hipErrorInvalidValue;
  int n = seq * (d / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (float2*)table, seq, d / 2, (double)base);
  return hipGetLastError();
}

hipError_t launch_rope(int dtype, const void* src, void* dst, const float* table, int rows, int seq, int n_q, int n_kv,
                       int d, int backward, int do_rotate, hipStream_t s) {
  if (rows <= 0 || seq <= 0) return hipErrorInvalidValue;
  const int vn = dtype == DT_BF16 ? 8 : 4;
  if ((d / 2) % vn) return hipErrorInvalidValue;
  const int n_rot = n_q + n_kv;
  const int hg = n_rot % 8 == 0 ? 8 : n_rot % 4 == 0 ? 4 : 1;            // heads per thread
  size_t items = (size_t)rows * (n_rot / hg) * (d / 2 / vn) + (src != dst ? (size_t)rows * n_kv * (d / vn) : 0);
  int g = grid_for(items, 256);
  float sign = backward ? -1.f : 1.f;
#define OPTSTAGE_ROPE(T, HG) \
  hipLaunchKernelGGL((rope_kernel<T, HG>), dim3(g), dim3(256), 0, s, (const T*)src, (T*)dst, (const float2*)table, rows, \
                     seq, n_rot, n_kv, d, sign, do_rotate)
  if (dtype == DT_BF16) { if (hg == 8) OPTSTAGE_ROPE(bf16_t, 8); else if (hg == 4) OPTSTAGE_ROPE(bf16_t, 4); else OPTSTAGE_ROPE(bf16_t, 1); }
  else { if (hg == 8) OPTSTAGE_ROPE(float, 8); else if (hg == 4) OPTSTAGE_ROPE(float, 4); else OPTSTAGE_ROPE(float, 1); }
#undef OPTSTAGE_ROPE
  return hipGetLastError();
}

hipError_t launch_slabs(const void* src, void* dst, int N, int K, int transposed, hipStream_t s) {
  if (N <= 0 || K <= 0 || (K % 64)) return hipErrorInvalidValue;
  const int n_pad = (N + 255) / 256 * 256;
  dim3 grid(K / 64, n_pad / 64);
  if (transposed == 2 && (N % 256)) return hipErrorInvalidValue;      // paired: N = 2 f with f a multiple of 128
  if (transposed == 1) hipLaunchKernelGGL(slab_kernel<true>, grid, dim3(256), 0, s, (const unsigned short*)src, (unsigned short*)dst, N, K, 0);
  else hipLaunchKernelGGL(slab_kernel<false>, grid, dim3(256), 0, s, (const unsigned short*)src, (unsigned short*)dst, N, K,
                          transposed == 2 ? N / 2 : 0);
  return hipGetLastError();
}

hipError_t launch_transpose(int dtype, const void* src, void* dst, int rows, int cols, hipStream_t s) {
  if (rows <= 0 || cols <= 0) return hipErrorInvalidValue;
  dim3 grid((cols + 63) / 64, (rows + 63) / 64);
  if (dtype == DT_BF16) hipLaunchKernelGGL(transpose_kernel<unsigned short>, grid, dim3(256), 0, s,
      (const unsigned short*)src, (unsigned short*)dst, rows, cols);
  else hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, s, (const float*)src, (float*)dst, rows, cols);
  return hipGetLastError();
}

hipError_t launch_checksum(const void* buf, uint64_t bytes, uint64_t* out_dev, hipStream_t s) {
  if (bytes % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(checksum_zero_kernel, dim3(1), dim3(1), 0, s, (unsigned long long*)out_dev);
  size_t n = bytes / 8;
  if (n) hipLaunchKernelGGL(checksum_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, (const unsigned long long*)buf, n,
      (unsigned long long*)out_dev);
  return hipGetLastError();
}
