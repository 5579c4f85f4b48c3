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

// LDS swizzles.  The LDS serves 16-byte reads 16 lanes at a time and 8-byte reads 32 lanes at a time over
// 64 four-byte banks (256 B), writes in 128-byte passes; each access pattern below touches every bank once.
// [rows][128] bf16 tile, 256 B per row: 16-byte chunk c of row r is stored at chunk c ^ (r & 15), so the
// 16 lanes that read one chunk of 16 consecutive rows hit 16 different chunks.
__device__ __forceinline__ int rowmajor_off(int r, int c) { return r * 256 + ((c ^ (r & 15)) << 4); }
// [128][64] bf16 transposed tile, 128 B per row: 8-byte granule q of row r is stored at granule
// q ^ (((r >> 3) ^ ((r & 7) << 1)) & 15): distinct over 16 consecutive rows, over (row parity, granule) of
// 32 consecutive rows (operand reads), and over rows 8 apart (the 16 lanes of one transposing store).
__device__ __forceinline__ int transposed_off(int r, int q) { return r * 128 + ((q ^ (((r >> 3) ^ ((r & 7) << 1)) & 15)) << 3); }

// Per-lane constants of the operand reads: every LDS address is (lane base) + (compile-time tile offset) +
// ((lane swizzle term) ^ (compile-time chunk term)), i.e. one xor-add per read.
struct FragAddr {
  int rm_base, rm_x, tr_base, tr_x;
  __device__ __forceinline__ FragAddr(int c32, int g) {
    rm_base = c32 * 256;
    rm_x = (g ^ (c32 & 15)) << 4;
    tr_base = c32 * 128;
    tr_x = ((((c32 >> 3) ^ ((c32 & 7) << 1)) & 15) ^ g) << 3;
  }
  // 16-byte operand of k-step ks (d = 16 ks + 8 g ..) from row 32 t + c32 of a row-major tile
  __device__ __forceinline__ bf16x8_t rowmajor(const char* lds, int t, int ks) const {
    return *reinterpret_cast<const bf16x8_t*>(lds + rm_base + 8192 * t + (rm_x ^ (ks << 5)));
  }
  // 8-element operand contracted over tile rows 32 t + 16 u + 4 g + {0..3} and + 8, column 32 dt + c32
  __device__ __forceinline__ bf16x8_t transposed(const char* lds, int dt, int t, int u) const {
    const int k = ((8 * t + 4 * u) ^ (4 * dt)) << 3;          // 4 dt enters the swizzle through row >> 3
    uint2 lo = *reinterpret_cast<const uint2*>(lds + tr_base + 4096 * dt + (tr_x ^ k));
    uint2 hi = *reinterpret_cast<const uint2*>(lds + tr_base + 4096 * dt + (tr_x ^ k ^ 16));
    uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
    return *reinterpret_cast<bf16x8_t*>(&v);
  }
};

// cooperative load of a [64 rows][128] tile (rows row0.., zero beyond nrows): thread (kq = tid / 16,
// dc = tid % 16) holds rows 4 kq .. 4 kq + 3 of 16-byte column chunk dc; the same registers feed both the
// row-major and the transposed LDS store
typedef int i32x4_t __attribute__((ext_vector_type(4)));
// Tiles are fetched with raw buffer loads: one 32-bit lane offset (row 4 kq, chunk dc) plus a scalar offset
// for (first row + kk, head); rows at or past the end of the tensor fall outside the buffer range and read
// as zero, so there is neither predication nor 64-bit address arithmetic in the loops.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ unsigned tile_lane_offset(int ld, int tid) { return (unsigned)((tid >> 4) * 4 * ld + (tid & 15) * 8) * 2u; }
// byte_off: scalar byte offset of (row0, first column of the head) inside the buffer
__device__ __forceinline__ void tile_load(uint4 reg[4], __amdgpu_buffer_rsrc_t rs, unsigned lane_off, unsigned byte_off, int ld) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    i32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, byte_off + (unsigned)(kk * ld * 2), 0);
    reg[kk] = make_uint4((unsigned)v[0], (unsigned)v[1], (unsigned)v[2], (unsigned)v[3]);
  }
}
__device__ __forceinline__ void tile_store_rowmajor(char* lds, const uint4 reg[4], int tid) {
  const int kq = tid >> 4, dc = tid & 15;
  const int base = kq * 1024, x = (dc ^ ((4 * kq) & 15)) << 4;      // row 4 kq + kk: (row & 15) = (4 kq & 15) ^ kk
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) *reinterpret_cast<uint4*>(lds + base + kk * 256 + (x ^ (kk << 4))) = reg[kk];
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
    // row 8 dc + i: swizzle term ((row >> 3) ^ ((row & 7) << 1)) & 15 = dc ^ 2 i
    *reinterpret_cast<uint2*>(lds + dc * 1024 + i * 128 + ((((kq ^ dc) & 15) << 3) ^ (i << 4))) = make_uint2(o[0], o[1]);
  }
}
__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& s, int u) {
  bf16x8_t r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)s[8 * u + e];
  return r;
}


// One 32 x 32 score tile (and optionally the matching dP tile) over the 8 k-steps of head_dim 128, with the
// LDS operand reads of k-step ks + 1 issued before the MFMAs of k-step ks and scheduling fences in between,
// so that at most two k-steps of operands are live (bounded registers, no spills); the second wave of the
// SIMD covers what LDS latency remains.  LA / LB say whether an operand comes from an LDS tile (row
// block ta / tb) or from the register-resident fragments ra / rb.
template <bool TWO, bool LA, bool LB>
__device__ __forceinline__ void score_tiles(const FragAddr& fr, const char* sA0, const char* sA1, int ta,
                                            const char* sB0, const char* sB1, int tb, const bf16x8_t* ra0,
                                            const bf16x8_t* ra1, const bf16x8_t* rb0, const bf16x8_t* rb1,
                                            f32x16_t& s, f32x16_t& dp) {
  bf16x8_t a0[2], b0[2], a1[2], b1[2];
  auto fetch = [&](int buf, int ks) {
    if (LA) { a0[buf] = fr.rowmajor(sA0, ta, ks); if (TWO) a1[buf] = fr.rowmajor(sA1, ta, ks); }
    if (LB) { b0[buf] = fr.rowmajor(sB0, tb, ks); if (TWO) b1[buf] = fr.rowmajor(sB1, tb, ks); }
  };
  fetch(0, 0);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (ks < 7) fetch((ks + 1) & 1, ks + 1);
    __builtin_amdgcn_sched_barrier(0);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(LA ? a0[ks & 1] : ra0[ks], LB ? b0[ks & 1] : rb0[ks], s, 0, 0, 0);
    if (TWO) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(LA ? a1[ks & 1] : ra1[ks], LB ? b1[ks & 1] : rb1[ks], dp, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// acc[dt] += T^T-fragment(dt, t, u) x packed tile, for the 4 row tiles of head_dim 128 and both 16-wide
// contraction halves u of one 32-wide tile t
__device__ __forceinline__ void accumulate_transposed(const FragAddr& fr, const char* sT, int t, const f32x16_t& w,
                                                      f32x16_t (&acc)[4]) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    bf16x8_t f[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) f[dt] = fr.transposed(sT, dt, t, u);
    const bf16x8_t pw = pack8(w, u);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[dt], pw, acc[dt], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ---- forward ------------------------------------------------------------------------------------------
// grid (ceil(seq / 128), n_q, batch); 4 waves x 32 query rows; key blocks of 64
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                        float* __restrict__ lse, int seq, int n_q, int n_kv) {
  __shared__ __attribute__((aligned(16))) char smem[2 * 16384];
  char* sK = smem;
  char* sV = smem + 16384;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const FragAddr fr(c32, g);
  const int nqb = (seq + 127) / 128;
  const int q0 = (nqb - 1 - (int)blockIdx.x) * 128;          // longest rows first
  const int a = blockIdx.y, b = blockIdx.z, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
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
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (unsigned)seq * ld * 2u);
  const unsigned lane_off = tile_lane_offset(ld, tid);
  const unsigned k_off = (unsigned)(n_q + kvh) * D * 2u, v_off = (unsigned)(n_q + n_kv + kvh) * D * 2u;
  tile_load(kreg, rs, lane_off, k_off, ld);
  tile_load(vreg, rs, lane_off, v_off, ld);
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    tile_store_rowmajor(sK, kreg, tid);
    tile_store_transposed(sV, vreg, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      const unsigned row_off = (unsigned)(64 * (kb + 1)) * ld * 2u;
      tile_load(kreg, rs, lane_off, row_off + k_off, ld);
      tile_load(vreg, rs, lane_off, row_off + v_off, ld);
    }
    if (64 * kb > wave_last_q) continue;                       // wave-uniform: block above this wave's diagonal
    f32x16_t s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[t][v] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        bf16x8_t kf = fr.rowmajor(sK, t, ks);
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
          bf16x8_t vf = fr.transposed(sV, dt, t, u);
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
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, int seq, int n_q, int n_kv) {
  __shared__ __attribute__((aligned(16))) char smem[3 * 16384];
  char* sK = smem;
  char* sV = smem + 16384;
  char* sKt = smem + 32768;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const FragAddr fr(c32, g);
  const int nqb = (seq + 127) / 128;
  const int q0 = (nqb - 1 - (int)blockIdx.x) * 128;
  const int a = blockIdx.y, b = blockIdx.z, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
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
  const __amdgpu_buffer_rsrc_t rs = make_rsrc(base, (unsigned)seq * ld * 2u);
  const unsigned lane_off = tile_lane_offset(ld, tid);
  const unsigned k_off = (unsigned)(n_q + kvh) * D * 2u, v_off = (unsigned)(n_q + n_kv + kvh) * D * 2u;
  tile_load(kreg, rs, lane_off, k_off, ld);
  tile_load(vreg, rs, lane_off, v_off, ld);
  for (int kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    tile_store_rowmajor(sK, kreg, tid);
    tile_store_rowmajor(sV, vreg, tid);
    tile_store_transposed(sKt, kreg, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      const unsigned row_off = (unsigned)(64 * (kb + 1)) * ld * 2u;
      tile_load(kreg, rs, lane_off, row_off + k_off, ld);
      tile_load(vreg, rs, lane_off, row_off + v_off, ld);
    }
    if (64 * kb > wave_last_q) continue;
    const bool diag = 64 * kb + 63 > q0 + 32 * wave;              // block touches the diagonal: mask
    // the two 32-key halves of the block one after the other, so only one S / dP tile is live at a time
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16_t s, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
      score_tiles<true, true, false>(fr, sK, sV, t, nullptr, nullptr, 0, nullptr, nullptr, qf, dof, s, dp);
      if (diag) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int key = 64 * kb + 32 * t + 8 * (v >> 2) + 4 * g + (v & 3);
          float p = __builtin_amdgcn_exp2f(fmaf(s[v], c, -Lc));
          if (key > qglob) p = 0.f;
          s[v] = p * (dp[v] - Dq);                                // dS^T
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], c, -Lc)) * (dp[v] - Dq);
      }
      accumulate_transposed(fr, sKt, t, s, acc);
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

// ---- backward, dK / dV: grid (ceil(seq / 128), n_kv, batch); query blocks of 64 ---------------------------
// 8 waves share the LDS tiles of one workgroup.  Waves 0-3 own dV of 32 keys each (S -> P -> dV^T += dO^T P)
// and stage the Q / dO tiles; waves 4-7 own dK of the same keys (S, dP -> dS -> dK^T += Q^T dS).  Each SIMD
// thus runs one dV wave and one dK wave whose MFMA and exp2 phases interleave, and both stay within 256
// VGPRs, so MFMA results are written to ordinary VGPRs (no accumulator-file copies).
__global__ __launch_bounds__(512) void attn_bwd_dkv_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16_t* __restrict__ dqkv, int seq, int n_q, int n_kv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // [K | V] of the workgroup's 128 keys (32 KB each, loaded once), [Q | dO | Q^T | dO^T] of the current
  // 64-query block (16 KB each), then lse*log2e and D for those queries
  char* sK = smem;
  char* sV = smem + 32768;
  char* sQ = smem + 65536;
  char* sDO = sQ + 16384;
  char* sQt = sQ + 32768;
  char* sDOt = sQ + 49152;
  float* sL = reinterpret_cast<float*>(sQ + 65536);
  float* sD = sL + 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c32 = lane & 31;
  const FragAddr fr(c32, g);
  const bool is_dk = wave >= 4;          // wave-uniform role
  const int kw = wave & 3;               // which 32 keys of the block
  const bool loader = !is_dk;            // waves 0-3 (threads 0..255) stage the tiles
  const int k0 = blockIdx.x * 128;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int ld = (n_q + 2 * n_kv) * D;
  const int ldo = n_q * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const int kglob = k0 + 32 * kw + c32;
  const __amdgpu_buffer_rsrc_t rs_qkv = make_rsrc(base, (unsigned)seq * ld * 2u);
  const __amdgpu_buffer_rsrc_t rs_do = make_rsrc(dout + (size_t)b * seq * ldo, (unsigned)seq * ldo * 2u);
  const unsigned lane_off_qkv = tile_lane_offset(ld, tid & 255), lane_off_do = tile_lane_offset(ldo, tid & 255);
  if (loader) {
    uint4 r0[4], r1[4];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const unsigned row_off = (unsigned)(k0 + 64 * half) * ld * 2u;
      tile_load(r0, rs_qkv, lane_off_qkv, row_off + (unsigned)(n_q + kvh) * D * 2u, ld);
      tile_load(r1, rs_qkv, lane_off_qkv, row_off + (unsigned)(n_q + n_kv + kvh) * D * 2u, ld);
      tile_store_rowmajor(sK + 16384 * half, r0, tid);
      tile_store_rowmajor(sV + 16384 * half, r1, tid);
    }
  }
  const float scale = rsqrtf((float)D), c = scale * LOG2E;
  f32x16_t acc[4];                        // dV^T (waves 0-3) or dK^T (waves 4-7): [d 128][32 keys]
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[dt][v] = 0.f;
  const int rep = n_q / n_kv;
  const int qb0 = k0 / 64, nqb = (seq + 63) / 64;
  const int wave_first_k = k0 + 32 * kw;
  const int iters = rep * (nqb - qb0);
  uint4 qreg[4], doreg[4];
  float lreg = 0.f, dreg = 0.f;
  auto issue_loads = [&](int it) {
    const int a = kvh * rep + it / (nqb - qb0);
    const int r0 = 64 * (qb0 + it % (nqb - qb0));
    tile_load(qreg, rs_qkv, lane_off_qkv, (unsigned)r0 * ld * 2u + (unsigned)a * D * 2u, ld);
    tile_load(doreg, rs_do, lane_off_do, (unsigned)r0 * ldo * 2u + (unsigned)a * D * 2u, ldo);
    if (tid < 64) {
      int r = min(r0 + tid, seq - 1);
      lreg = lse[((size_t)b * n_q + a) * seq + r] * LOG2E;
      dreg = delta[((size_t)b * n_q + a) * seq + r];
    }
  };
  if (loader && iters > 0) issue_loads(0);
  for (int it = 0; it < iters; ++it) {
    const int r0 = 64 * (qb0 + it % (nqb - qb0));
    __syncthreads();
    if (loader) {
      tile_store_rowmajor(sQ, qreg, tid);
      tile_store_rowmajor(sDO, doreg, tid);
      tile_store_transposed(sQt, qreg, tid);
      tile_store_transposed(sDOt, doreg, tid);
      if (tid < 64) { sL[tid] = lreg; sD[tid] = dreg; }
    }
    __syncthreads();
    if (loader && it + 1 < iters) issue_loads(it + 1);
    if (r0 + 63 < wave_first_k) continue;                      // wave-uniform: all queries precede this wave's keys
    // lane = key (column), registers = queries: row v of tile t is query r0 + 32 t + 8 (v / 4) + 4 g + v % 4
    const bool edge = r0 < wave_first_k + 32 || r0 + 64 > seq;   // wave-uniform: diagonal or ragged tail
    if (!is_dk) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16_t s, unused;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
        score_tiles<false, true, true>(fr, sQ, nullptr, t, sK, nullptr, kw, nullptr, nullptr, nullptr, nullptr, s, unused);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ql0 = 32 * t + 8 * j + 4 * g;
          const f32x4_t L4 = *reinterpret_cast<const f32x4_t*>(sL + ql0);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = 4 * j + i;
            float p = __builtin_amdgcn_exp2f(fmaf(s[v], c, -L4[i]));
            if (edge) {
              const int qg = r0 + ql0 + i;
              if (qg < kglob || qg >= seq) p = 0.f;
            }
            s[v] = p;
          }
        }
        accumulate_transposed(fr, sDOt, t, s, acc);
      }
    } else {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x16_t s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
        score_tiles<true, true, true>(fr, sQ, sDO, t, sK, sV, kw, nullptr, nullptr, nullptr, nullptr, s, dp);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int ql0 = 32 * t + 8 * j + 4 * g;
          const f32x4_t L4 = *reinterpret_cast<const f32x4_t*>(sL + ql0);
          const f32x4_t D4 = *reinterpret_cast<const f32x4_t*>(sD + ql0);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = 4 * j + i;
            float p = __builtin_amdgcn_exp2f(fmaf(s[v], c, -L4[i]));
            if (edge) {
              const int qg = r0 + ql0 + i;
              if (qg < kglob || qg >= seq) p = 0.f;
            }
            s[v] = p * (dp[v] - D4[i]);                           // dS
          }
        }
        accumulate_transposed(fr, sQt, t, s, acc);
      }
    }
  }
  if (kglob >= seq) return;
  const float osc = is_dk ? scale : 1.f;
  bf16_t* orow = dqkv + ((size_t)b * seq + kglob) * ld + (size_t)(is_dk ? n_q + kvh : n_q + n_kv + kvh) * D;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x4_t r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (bf16_t)(acc[dt][4 * j + i] * osc);
      *reinterpret_cast<bf16x4_t*>(orow + 32 * dt + 8 * j + 4 * g) = r;
    }
}

}  // namespace

// bf16, head_dim 128, and per-sequence tensors addressable with 32-bit byte offsets (buffer loads)
bool attn_mfma_applies(int dtype, int d, int seq, int n_q, int n_kv) {
  return dtype == DT_BF16 && d == 128 && (unsigned long long)(seq + 256) * (n_q + 2 * n_kv) * 128 * 2 < 0xF0000000ull;
}

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
  constexpr int smem = 2 * 32768 + 65536 + 512;
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_mfma), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(attn_bwd_dkv_mfma, dim3((seq + 127) / 128, n_kv, batch), dim3(512), smem, s, (const bf16_t*)qkv, (const bf16_t*)dout, lse, ws, (bf16_t*)dqkv, seq, n_q, n_kv);
  return hipGetLastError();
}
