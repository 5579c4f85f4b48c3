// Fused causal attention, bf16 MFMA path for head_dim 128 (gfx950): forward (online softmax, writes
// lse) and backward (dQ kernel + dK/dV kernel, both recomputing the probabilities from lse; no atomics,
// so results are bitwise reproducible).  q-head a reads kv-head a * n_kv / n_q; dK, dV are summed over
// the q-heads of a group inside the dK/dV kernel.
//
// Register / LDS scheme.  Every product is issued on v_mfma_f32_32x32x16_bf16 in the orientation whose
// accumulator layout (one column per lane, 4-row groups along registers) already has the shape of the
// next product's 8-element operand, so probabilities never move between lanes:
//   forward / dQ:  S^T = K Q^T (lane = query, registers = keys)  ->  O^T += V^T P^T,  dQ^T += K^T dS^T
//   dK/dV:         S   = Q K^T (lane = key,   registers = queries) -> dV^T += dO^T P,  dK^T += Q^T dS
// Operands that are contracted over their row index (V^T, K^T, dO^T, Q^T) are transposed in registers on
// the way into LDS (4 x 8 patches, 8-byte stores); all LDS tiles are XOR-swizzled so that operand reads
// and tile writes are bank-conflict free.
#include "common.h"

namespace {

constexpr int D = 128;
constexpr float LOG2E = 1.4426950408889634f;

// [rows][128] bf16 tile, 256 B per row, 16-byte chunk c of row r stored at chunk c ^ (r & 7)
__device__ __forceinline__ int rowmajor_off(int r, int c) { return r * 256 + ((c ^ (r & 7)) << 4); }
// [128][64] bf16 transposed tile, 128 B per row, 8-byte granule q of row r stored at granule
// q ^ ((r ^ (r >> 3)) & 15): distinct for 16 consecutive rows (operand reads) and for rows 8 apart (tile writes)
__device__ __forceinline__ int transposed_off(int r, int q) { return r * 128 + ((q ^ ((r ^ (r >> 3)) & 15)) << 3); }

// cooperative load of a [64 rows][128] tile (rows row0.., zero beyond nrows): thread (kq = tid / 16,
// dc = tid % 16) holds rows 4 kq .. 4 kq + 3 of 16-byte column chunk dc; the same registers feed both the
// row-major and the transposed LDS store
__device__ __forceinline__ void tile_load(uint4 reg[4], const bf16_t* p, int ld, int row0, int nrows, int tid) {
  const int kq = tid >> 4, dc = tid & 15;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    int r = row0 + 4 * kq + kk;
    reg[kk] = (r < nrows) ? *reinterpret_cast<const uint4*>(p + (size_t)r * ld + dc * 8) : make_uint4(0, 0, 0, 0);
  }
}
__device__ __forceinline__ void tile_store_rowmajor(char* lds, const uint4 reg[4], int tid) {
  const int kq = tid >> 4, dc = tid & 15;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) *reinterpret_cast<uint4*>(lds + rowmajor_off(4 * kq + kk, dc)) = reg[kk];
}
__device__ __forceinline__ void tile_store_transposed(char* lds, const uint4 reg[4], int tid) {
  const int kq = tid >> 4, dc = tid & 15;
  const uint32_t* w = reinterpret_cast<const uint32_t*>(reg);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint32_t o[2];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      uint32_t a = w[(2 * pr) * 4 + (i >> 1)], b = w[(2 * pr + 1) * 4 + (i >> 1)];
      o[pr] = (i & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
    }
    *reinterpret_cast<uint2*>(lds + transposed_off(dc * 8 + i, kq)) = make_uint2(o[0], o[1]);
  }
}
// 8-element operand contracted over tile rows: rows 4 q1 .. +3 and 4 (q1 + 2) .. +3 of column r
__device__ __forceinline__ bf16x8_t read_transposed_frag(const char* lds, int r, int q1) {
  uint2 lo = *reinterpret_cast<const uint2*>(lds + transposed_off(r, q1));
  uint2 hi = *reinterpret_cast<const uint2*>(lds + transposed_off(r, q1 + 2));
  uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
  return *reinterpret_cast<bf16x8_t*>(&v);
}
__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& s, int u) {
  bf16x8_t r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)s[8 * u + e];
  return r;
}

// ---- forward ------------------------------------------------------------------------------------------
// grid (ceil(seq / 128), n_q, batch); 4 waves x 32 query rows; key blocks of 64
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                        float* __restrict__ lse, int seq, int n_q, int n_kv) {
  __shared__ __attribute__((aligned(16))) char smem[2 * 16384];
  char* sK = smem;
  char* sV = smem + 16384;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const int nqb = (seq + 127) / 128;
  const int q0 = (nqb - 1 - (int)blockIdx.x) * 128;          // longest rows first
  const int a = blockIdx.y, b = blockIdx.z, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const bf16_t* Kp = base + (size_t)(n_q + kvh) * D;
  const bf16_t* Vp = base + (size_t)(n_q + n_kv + kvh) * D;
  const int qglob = q0 + 32 * wave + c32;
  const int qrow = min(qglob, seq - 1);
  bf16x8_t qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)qrow * ld + a * D + 16 * ks + 8 * g);
  f32x16_t oacc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float scale = rsqrtf((float)D), c = scale * LOG2E;
  const int nkb = min((q0 + 127) / 64 + 1, (seq + 63) / 64);
  const int wave_last_q = q0 + 32 * wave + 31;
  uint4 kreg[4], vreg[4];
  tile_load(kreg, Kp, ld, 0, seq, tid);
  tile_load(vreg, Vp, ld, 0, seq, tid);
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    tile_store_rowmajor(sK, kreg, tid);
    tile_store_transposed(sV, vreg, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      tile_load(kreg, Kp, ld, 64 * (kb + 1), seq, tid);
      tile_load(vreg, Vp, ld, 64 * (kb + 1), seq, tid);
    }
    if (64 * kb > wave_last_q) continue;                       // wave-uniform: block above this wave's diagonal
    f32x16_t s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sK + rowmajor_off(32 * t + c32, 2 * ks + g));
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[t], 0, 0, 0);
      }
    if (64 * kb + 63 > q0 + 32 * wave) {                       // block touches the diagonal
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int key = 64 * kb + 32 * t + 8 * (v >> 2) + 4 * g + (v & 3);
          if (key > qglob) s[t][v] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[t][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f((m - mn) * c);
    const float mc = mn * c;
    float ls = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], c, -mc));
        s[t][v] = p;
        ls += p;
      }
    l = l * alpha + ls;
    m = mn;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8_t pf = pack8(s[t], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          bf16x8_t vf = read_transposed_frag(sV, 32 * dt + c32, 8 * t + 4 * u + g);
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[dt], 0, 0, 0);
        }
      }
  }
  const float lt = l + __shfl_xor(l, 32, 64);
  if (qglob >= seq) return;
  const float inv = 1.f / lt;
  bf16_t* orow = o + ((size_t)b * seq + qglob) * (n_q * D) + a * D;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4_t r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (bf16_t)(oacc[dt][4 * j + i] * inv);
      *reinterpret_cast<bf16x4_t*>(orow + 32 * dt + 8 * j + 4 * g) = r;
    }
  if (g == 0) lse[((size_t)b * n_q + a) * seq + qglob] = m * scale + logf(lt);
}

// ---- backward, step 0: D_t = <dO_t, O_t> per query row and head ----------------------------------------
__global__ void attn_bwd_delta(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout, float* __restrict__ delta,
                               int seq, int n_q, int batch) {
  // one wave per (row, head): 64 lanes x 2 elements
  const int lane = threadIdx.x & 63;
  const size_t w = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const size_t total = (size_t)batch * seq * n_q;
  if (w >= total) return;
  const size_t row = w / n_q;
  const int a = w % n_q;
  const size_t off = row * ((size_t)n_q * D) + (size_t)a * D + 2 * lane;
  float s = (float)o[off] * (float)dout[off] + (float)o[off + 1] * (float)dout[off + 1];
  s = wave_sum(s);
  const int b = row / seq, t = row % seq;
  if (lane == 0) delta[((size_t)b * n_q + a) * seq + t] = s;
}

// ---- backward, dQ: grid (ceil(seq / 128), n_q, batch); 4 waves x 32 query rows; key blocks of 64 ---------
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, int seq, int n_q, int n_kv) {
  __shared__ __attribute__((aligned(16))) char smem[3 * 16384];
  char* sK = smem;
  char* sV = smem + 16384;
  char* sKt = smem + 32768;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const int nqb = (seq + 127) / 128;
  const int q0 = (nqb - 1 - (int)blockIdx.x) * 128;
  const int a = blockIdx.y, b = blockIdx.z, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const bf16_t* Kp = base + (size_t)(n_q + kvh) * D;
  const bf16_t* Vp = base + (size_t)(n_q + n_kv + kvh) * D;
  const int qglob = q0 + 32 * wave + c32;
  const int qrow = min(qglob, seq - 1);
  const bf16_t* dop = dout + ((size_t)b * seq + qrow) * (n_q * D) + a * D;
  bf16x8_t qf[8], dof[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)qrow * ld + a * D + 16 * ks + 8 * g);
    dof[ks] = *reinterpret_cast<const bf16x8_t*>(dop + 16 * ks + 8 * g);
  }
  const float scale = rsqrtf((float)D), c = scale * LOG2E;
  const float Lc = lse[((size_t)b * n_q + a) * seq + qrow] * LOG2E;
  const float Dq = delta[((size_t)b * n_q + a) * seq + qrow];
  f32x16_t acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;
  const int nkb = min((q0 + 127) / 64 + 1, (seq + 63) / 64);
  const int wave_last_q = q0 + 32 * wave + 31;
  uint4 kreg[4], vreg[4];
  tile_load(kreg, Kp, ld, 0, seq, tid);
  tile_load(vreg, Vp, ld, 0, seq, tid);
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    tile_store_rowmajor(sK, kreg, tid);
    tile_store_rowmajor(sV, vreg, tid);
    tile_store_transposed(sKt, kreg, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      tile_load(kreg, Kp, ld, 64 * (kb + 1), seq, tid);
      tile_load(vreg, Vp, ld, 64 * (kb + 1), seq, tid);
    }
    if (64 * kb > wave_last_q) continue;
    f32x16_t s[2], dp[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[t][v] = 0.f; dp[t][v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sK + rowmajor_off(32 * t + c32, 2 * ks + g));
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[t], 0, 0, 0);
        bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(sV + rowmajor_off(32 * t + c32, 2 * ks + g));
        dp[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[ks], dp[t], 0, 0, 0);
      }
    const bool diag = 64 * kb + 63 > q0 + 32 * wave;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int key = 64 * kb + 32 * t + 8 * (v >> 2) + 4 * g + (v & 3);
        float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], c, -Lc));
        if (diag && key > qglob) p = 0.f;
        s[t][v] = p * (dp[t][v] - Dq);                            // dS^T
      }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8_t df = pack8(s[t], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          bf16x8_t kt = read_transposed_frag(sKt, 32 * dt + c32, 8 * t + 4 * u + g);
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, df, acc[dt], 0, 0, 0);
        }
      }
  }
  if (qglob >= seq) return;
  bf16_t* dq = dqkv + ((size_t)b * seq + qglob) * ld + a * D;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4_t r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (bf16_t)(acc[dt][4 * j + i] * scale);
      *reinterpret_cast<bf16x4_t*>(dq + 32 * dt + 8 * j + 4 * g) = r;
    }
}

// ---- backward, dK / dV: grid (ceil(seq / 128), n_kv, batch); 4 waves x 32 keys; query blocks of 64 -------
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16_t* __restrict__ dqkv, int seq, int n_q, int n_kv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // [Q | dO | Q^T | dO^T] 16 KB each, then lse*log2e and D for the 64 queries of the block
  char* sQ = smem;
  char* sDO = smem + 16384;
  char* sQt = smem + 32768;
  char* sDOt = smem + 49152;
  float* sL = reinterpret_cast<float*>(smem + 65536);
  float* sD = sL + 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const int k0 = blockIdx.x * 128;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int ld = (n_q + 2 * n_kv) * D;
  const int ldo = n_q * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const int kglob = k0 + 32 * wave + c32;
  const int krow = min(kglob, seq - 1);
  bf16x8_t kf[8], vf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)krow * ld + (n_q + kvh) * D + 16 * ks + 8 * g);
    vf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)krow * ld + (n_q + n_kv + kvh) * D + 16 * ks + 8 * g);
  }
  const float scale = rsqrtf((float)D), c = scale * LOG2E;
  f32x16_t dk[4], dv[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
  const int rep = n_q / n_kv;
  const int qb0 = k0 / 64, nqb = (seq + 63) / 64;
  const int wave_first_k = k0 + 32 * wave;
  const int iters = rep * (nqb - qb0);
  uint4 qreg[4], doreg[4];
  float lreg = 0.f, dreg = 0.f;
  auto issue_loads = [&](int it) {
    const int a = kvh * rep + it / (nqb - qb0);
    const int r0 = 64 * (qb0 + it % (nqb - qb0));
    const bf16_t* Qp = base + (size_t)a * D;
    const bf16_t* DOp = dout + (size_t)b * seq * ldo + (size_t)a * D;
    tile_load(qreg, Qp, ld, r0, seq, tid);
    tile_load(doreg, DOp, ldo, r0, seq, tid);
    if (tid < 64) {
      int r = min(r0 + tid, seq - 1);
      lreg = lse[((size_t)b * n_q + a) * seq + r] * LOG2E;
      dreg = delta[((size_t)b * n_q + a) * seq + r];
    }
  };
  if (iters > 0) issue_loads(0);
  for (int it = 0; it < iters; ++it) {
    const int r0 = 64 * (qb0 + it % (nqb - qb0));
    __syncthreads();
    tile_store_rowmajor(sQ, qreg, tid);
    tile_store_rowmajor(sDO, doreg, tid);
    tile_store_transposed(sQt, qreg, tid);
    tile_store_transposed(sDOt, doreg, tid);
    if (tid < 64) { sL[tid] = lreg; sD[tid] = dreg; }
    __syncthreads();
    if (it + 1 < iters) issue_loads(it + 1);
    if (r0 + 63 < wave_first_k) continue;                      // wave-uniform: all queries precede this wave's keys
    f32x16_t s[2], dp[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[t][v] = 0.f; dp[t][v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8_t qf = *reinterpret_cast<const bf16x8_t*>(sQ + rowmajor_off(32 * t + c32, 2 * ks + g));
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ks], s[t], 0, 0, 0);
        bf16x8_t dof = *reinterpret_cast<const bf16x8_t*>(sDO + rowmajor_off(32 * t + c32, 2 * ks + g));
        dp[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dof, vf[ks], dp[t], 0, 0, 0);
      }
    // lane = key (column), registers = queries: row r of tile t is query r0 + 32 t + 8 (v / 4) + 4 g + v % 4
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int ql = 32 * t + 8 * (v >> 2) + 4 * g + (v & 3);
        const int qg = r0 + ql;
        float p = __builtin_amdgcn_exp2f(fmaf(s[t][v], c, -sL[ql]));
        if (qg < kglob || qg >= seq) p = 0.f;
        dp[t][v] = p * (dp[t][v] - sD[ql]);                       // dS
        s[t][v] = p;
      }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        bf16x8_t pf = pack8(s[t], u), df = pack8(dp[t], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          bf16x8_t dot = read_transposed_frag(sDOt, 32 * dt + c32, 8 * t + 4 * u + g);
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, pf, dv[dt], 0, 0, 0);
          bf16x8_t qt = read_transposed_frag(sQt, 32 * dt + c32, 8 * t + 4 * u + g);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, df, dk[dt], 0, 0, 0);
        }
      }
  }
  if (kglob >= seq) return;
  bf16_t* dkr = dqkv + ((size_t)b * seq + kglob) * ld + (n_q + kvh) * D;
  bf16_t* dvr = dqkv + ((size_t)b * seq + kglob) * ld + (n_q + n_kv + kvh) * D;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4_t rk, rv;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        rk[i] = (bf16_t)(dk[dt][4 * j + i] * scale);
        rv[i] = (bf16_t)dv[dt][4 * j + i];
      }
      *reinterpret_cast<bf16x4_t*>(dkr + 32 * dt + 8 * j + 4 * g) = rk;
      *reinterpret_cast<bf16x4_t*>(dvr + 32 * dt + 8 * j + 4 * g) = rv;
    }
}

}  // namespace

bool attn_mfma_applies(int dtype, int d) { return dtype == DT_BF16 && d == 128; }

hipError_t launch_attn_fwd_mfma(const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv, hipStream_t s) {
  hipLaunchKernelGGL(attn_fwd_mfma, dim3((seq + 127) / 128, n_q, batch), dim3(256), 0, s, (const bf16_t*)qkv, (bf16_t*)o, lse, seq, n_q, n_kv);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv, float* ws,
                                int seq, int batch, int n_q, int n_kv, hipStream_t s) {
  const size_t rows = (size_t)batch * seq * n_q;
  hipLaunchKernelGGL(attn_bwd_delta, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, (const bf16_t*)o, (const bf16_t*)dout, ws, seq, n_q, batch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_mfma, dim3((seq + 127) / 128, n_q, batch), dim3(256), 0, s, (const bf16_t*)qkv, (const bf16_t*)dout, lse, ws, (bf16_t*)dqkv, seq, n_q, n_kv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr int smem = 65536 + 512;
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_mfma), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_bwd_dkv_mfma, dim3((seq + 127) / 128, n_kv, batch), dim3(256), smem, s, (const bf16_t*)qkv, (const bf16_t*)dout, lse, ws, (bf16_t*)dqkv, seq, n_q, n_kv);
  return hipGetLastError();
}
