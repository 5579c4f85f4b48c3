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
// Tiles go from global memory straight into LDS, row-major; operands that are contracted over their row
// index (V^T, K^T, dO^T, Q^T) come out of the same tile through transposing LDS reads.  All LDS tiles are
// XOR-swizzled so that both kinds of operand reads are bank-conflict free.
#include "common.h"

namespace {

constexpr int D = 128;
constexpr float LOG2E = 1.4426950408889634f;

typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& s, int u) {
  bf16x8_t r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)s[8 * u + e];
  return r;
}

// max over the two lanes 32 apart (the two halves of a score row), in both of them: v_permlane32_swap exchanges
// the upper half of its first operand with the lower half of its second, so swapping x with itself gives
// (x.low, x.low) and (x.high, x.high).  A vector instruction: no trip through the LDS crossbar.
__device__ __forceinline__ float pair_max32(float x) {
  const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}

// ---- forward: grid (n_q, batch, ceil(seq / 256)); 4 waves (one per SIMD) ---------------------------------
// Same frame as the dQ kernel below: wave w owns queries q0 + 64 w .. + 63 as two 32-query tiles, Q operand
// fragments in registers, O^T ([d 128][64 queries]) in accumulator registers, key blocks of 64 (K and V rows)
// streaming through an LDS ring filled straight from global memory (three stages: the scores of the next
// block's first tile are issued before the current block's last tile is finished).  Per 32-key tile:
//   S^T = K Q^T (16 MFMAs), p = exp2(c s - c m_ref) with row sums, O^T += V^T P^T (16 MFMAs, V^T through
//   transposing LDS reads of the row-major V tile).
// One wave per SIMD means nothing else hides the exponentials (v_exp_f32 runs at a quarter of the vector rate:
// per tile they cost about half of what the 32 MFMAs cost), so the steps of consecutive tiles are interleaved by
// hand: the exponentials of tile i run between the score MFMAs of tile i + 1, the row maxima of tile i + 1
// between the O^T MFMAs of tile i.
// The softmax reference m_ref is not the running maximum: it is raised (and O^T and the row sums rescaled)
// only when some row of the wave finds a score more than FWD_TAU / c above it, so p <= 2^FWD_TAU and the
// rescaling, which would sit between consecutive tiles' MFMAs on the same accumulators, is rare after the first
// tiles.  softmax does not depend on the reference: o = (sum p v) / (sum p), lse = m_ref scale + log(sum p).
constexpr int FWD_STAGE = 32768;             // K tile, V tile of 64 keys
constexpr int FWD_SMEM = 3 * FWD_STAGE;
constexpr float FWD_TAU = 8.f;

__global__ __launch_bounds__(256) void attn_fwd_mfma(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                     float* __restrict__ lse, int seq, int n_q, int n_kv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqb = (seq + 255) / 256;
  const int q0 = (nqb - 1 - (int)blockIdx.z) * 256;          // longest rows are dispatched first, for every head
  const int a = blockIdx.x, b = blockIdx.y, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D, ldo = n_q * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const int wave_first_q = q0 + 64 * wave, wave_last_q = wave_first_q + 63;
  const float scale = rsqrtf((float)D), c = scale * LOG2E, thr = FWD_TAU / c;

  bf16x8_t Qf[2][8];
  int qglob[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    qglob[qt] = wave_first_q + 32 * qt + c32;
    const bf16_t* qp = base + (size_t)min(qglob[qt], seq - 1) * ld + (size_t)a * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) Qf[qt][ks] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * ks);
  }
  f32x16_t acc[2][4];                          // [query tile][d tile]: lane = query, registers = d
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][dt][v] = 0.f;
  float mref[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};

  // LDS addressing as in the dQ kernel: 64 rows x 256 B per tile, 16-byte chunk c of row r stored at chunk
  // c ^ (((r & 3) << 2) | ((r >> 2) & 3))
  int rm_addr[8];
  {
    const int f = ((c32 & 3) << 2) | ((c32 >> 2) & 3);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) rm_addr[ks] = c32 * 256 + (((2 * ks + g) ^ f) << 4);
  }
  int tr_addr[4][2];
  {
    const int cg = (lane >> 4) & 1, e = (lane >> 2) & 3, r = lane & 3;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int kq = 0; kq < 2; ++kq)
        tr_addr[dt][kq] = (4 * g + e) * 256 + (((4 * dt + 2 * cg + (r >> 1)) ^ (e << 2) ^ g ^ (kq << 1)) << 4) + (r & 1) * 8;
  }
  unsigned voff[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = 16 * wave + 4 * j + (lane >> 4);
    const int chunk = (lane & 15) ^ (((lane >> 4) << 2) | j);
    voff[j] = (unsigned)row * (unsigned)ld * 2u + (unsigned)chunk * 16u;
  }
  i32x4_t rs;
  {
    const unsigned long long ad = (unsigned long long)base;
    rs[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)ad);
    rs[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(ad >> 32) & 0xffff);
    rs[2] = (int)((unsigned)seq * ld * 2u);                   // rows at or past seq read zero
    rs[3] = 0x00020000;
  }
  const unsigned lds0 = (unsigned)(size_t)(lds_void_t*)smem;
  const unsigned k_off = (unsigned)(n_q + kvh) * D * 2u, v_off = (unsigned)(n_q + n_kv + kvh) * D * 2u;
  auto issue_block = [&](int kb, int stage) {
    const unsigned rowoff = (unsigned)(64 * kb) * (unsigned)ld * 2u;
    const unsigned dst = lds0 + stage * FWD_STAGE + (16 * wave) * 256;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + j * 1024), "v"(voff[j] + rowoff + k_off), "s"(rs) : "memory", "m0");
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + 16384 + j * 1024), "v"(voff[j] + rowoff + v_off), "s"(rs) : "memory", "m0");
    }
  };
  typedef short i16x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
  auto tr_frag = [&](const char* tile, int dt, int t, int u) {
    const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u) * 256 + tr_addr[dt][0]));
    const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u + 8) * 256 + tr_addr[dt][1]));
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto rm_frag = [&](const char* tile, int t, int ks) {
    return *reinterpret_cast<const bf16x8_t*>(tile + t * 8192 + rm_addr[ks]);
  };

  const int nkb = min((q0 + 255) / 64 + 1, (seq + 63) / 64);

#define OPTSTAGE_SB() __builtin_amdgcn_sched_barrier(0)
#define OPTSTAGE_MFMA_V(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
  // O^T and the Q fragments stay in the accumulation half of the register file (an MFMA takes its A / B operands
  // from either half): the vector half holds two score tiles, the streaming operand fragments and addresses.  A
  // compiler-chosen form would shuttle O^T between the halves at every tile.
#define OPTSTAGE_MFMA_A(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b))
  // Every wave runs every tile of the workgroup's 2 nkb, with no branch around a step: a tile above a wave's
  // diagonal is masked entirely (p = 0 adds nothing), and its SIMD would wait for the workgroup's last wave
  // anyway.  The scores issued in the very last step read a stage that holds no tile of this workgroup's; they
  // are never used.
  //
  // scores of the next tile into nxt (K half t of the tile in `stage_k`), between them the exponentials of the
  // current tile in cur
  // The first operand fragment of every step is read during the step before it (kf_first, trf_first), so that no
  // step starts with the matrix unit idle for an LDS round trip.
  bf16x8_t kf_first, trf_first;
  auto step_scores = [&](bool with_exp, int stage_k, int t, f32x16_t (&cur)[2], f32x16_t (&nxt)[2], int stage_v, int tv) {
    const char* sK = smem + stage_k * FWD_STAGE;
    bf16x8_t kf[2];
    kf[0] = kf_first;
    const float mc0 = mref[0] * c, mc1 = mref[1] * c;
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      OPTSTAGE_SB();
      if (ks < 7) kf[(ks + 1) & 1] = rm_frag(sK, t, ks + 1);
      else trf_first = tr_frag(smem + stage_v * FWD_STAGE + 16384, 0, tv, 0);
      OPTSTAGE_SB();
      // The compiler does not see into the MFMA statements, so it keeps no distance between a vector instruction
      // that produces an operand (a copy, a read of an accumulation register that holds part of Q) and the MFMA
      // that consumes it: have the operands in place, then two idle cycles
      asm volatile("s_nop 1" :: "v"(kf[ks & 1]));
      // One MFMA, then vector work for about as long as it occupies the matrix unit, then the next: a wave that
      // reaches an MFMA while the unit is busy waits there and issues nothing else, so two MFMAs back to back
      // followed by all of the vector work run one after the other instead of side by side.
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        if (ks == 0)                                             // the first k-step starts from C = 0
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(nxt[qt]) : "v"(kf[0]), "a"(Qf[qt][0]));
        else
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(nxt[qt]) : "v"(kf[ks & 1]), "a"(Qf[qt][ks]));
        OPTSTAGE_SB();
        if (with_exp) {                                          // compile-time after inlining
          const int v = 2 * ks + qt;
          const float p0 = __builtin_amdgcn_exp2f(fmaf(cur[0][v], c, -mc0));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(cur[1][v], c, -mc1));
          cur[0][v] = p0; cur[1][v] = p1;
          ls0 += p0; ls1 += p1;
          // keeps these instructions here, between the MFMAs: without a use at this point the compiler sinks
          // them to where the probabilities are packed
          asm volatile("" : "+v"(cur[0][v]), "+v"(cur[1][v]), "+v"(ls0), "+v"(ls1));
        }
        OPTSTAGE_SB();
      }
    }
    OPTSTAGE_SB();
    lsum[0] += ls0; lsum[1] += ls1;
  };
  // scores above the diagonal (and keys past the sequence, which lie above every stored query) leave the softmax
  auto mask_tile = [&](int i, f32x16_t (&sc)[2]) {
    if (32 * i + 31 <= wave_first_q) return;                     // wave-uniform: the tile lies below the diagonal
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * i + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
      for (int qt = 0; qt < 2; ++qt)
        if (key > qglob[qt]) sc[qt][v] = -INFINITY;
    }
  };
  auto max_half = [&](int n, int qt, const f32x16_t (&sc)[2], float (&mx)[2]) {
    mx[qt] = fmaxf(mx[qt], fmaxf(sc[qt][2 * n], sc[qt][2 * n + 1]));
    asm volatile("" : "+v"(mx[qt]));                            // stays between the MFMAs it is written between
  };
  auto max_slice = [&](int n, const f32x16_t (&sc)[2], float (&mx)[2]) {
    mx[0] = fmaxf(mx[0], fmaxf(sc[0][2 * n], sc[0][2 * n + 1]));
    mx[1] = fmaxf(mx[1], fmaxf(sc[1][2 * n], sc[1][2 * n + 1]));
    asm volatile("" : "+v"(mx[0]), "+v"(mx[1]));               // stays between the MFMAs it is written between
  };
  // the rare raise of m_ref, with O^T and the row sums rescaled
  auto raise_reference = [&](float (&mx)[2]) {
    mx[0] = pair_max32(mx[0]);                                  // the two lanes of a row hold 16 keys each
    mx[1] = pair_max32(mx[1]);
    if (__any((mx[0] > mref[0] + thr) | (mx[1] > mref[1] + thr))) {
      asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");         // the last O^T MFMAs have left the matrix unit
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const float mn = fmaxf(mref[qt], mx[qt]);
        const float alpha = mn == mref[qt] ? 1.f : __builtin_amdgcn_exp2f((mref[qt] - mn) * c);
        mref[qt] = mn;
        lsum[qt] *= alpha;
        // one accumulator tile at a time: they pass through vector registers for the multiplication
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          OPTSTAGE_SB();
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[qt][dt][v] *= alpha;
        }
        OPTSTAGE_SB();
      }
    }
  };
  // O^T += V^T P^T of the current tile (probabilities in cur, V half t of the tile in `stage_v`), between the MFMAs
  // the row maxima of the next tile i1 (scores in nxt, already masked)
  auto step_output = [&](int stage_v, int t, int i1, f32x16_t (&cur)[2], f32x16_t (&nxt)[2], int stage_k, int tk) {
    const char* sV = smem + stage_v * FWD_STAGE + 16384;
    mask_tile(i1, nxt);
    float mx[2] = {-INFINITY, -INFINITY};
    // fragment n + 2 is requested before the MFMAs of fragment n: one pair of MFMAs is shorter than an LDS round
    // trip
    bf16x8_t trf[3];
    trf[0] = trf_first;
    trf[1] = tr_frag(sV, 1, t, 0);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const bf16x8_t p0 = pack8(cur[0], u), p1 = pack8(cur[1], u);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const int n = u * 4 + dt, n2 = n + 2;
        OPTSTAGE_SB();
        if (n2 < 8) trf[n2 % 3] = tr_frag(sV, n2 & 3, t, n2 >> 2);
        else if (n == 6) kf_first = rm_frag(smem + stage_k * FWD_STAGE, tk, 0);
        if (dt == 0) asm volatile("s_nop 1" :: "v"(p0), "v"(p1) : "memory");   // packed operands settled
        OPTSTAGE_SB();
        OPTSTAGE_MFMA_A(acc[0][dt], trf[n % 3], p0);
        OPTSTAGE_SB();
        max_half(n, 0, nxt, mx);
        OPTSTAGE_SB();
        OPTSTAGE_MFMA_A(acc[1][dt], trf[n % 3], p1);
        OPTSTAGE_SB();
        max_half(n, 1, nxt, mx);
      }
    }
    OPTSTAGE_SB();
    raise_reference(mx);
  };
#define OPTSTAGE_BLOCK_SYNC() asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory")

  f32x16_t sA[2], sB[2];
  issue_block(0, 0);
  OPTSTAGE_BLOCK_SYNC();
  if (nkb > 1) issue_block(1, 1);
  kf_first = rm_frag(smem, 0, 0);
  step_scores(false, 0, 0, sB, sA, 0, 0);                      // scores of tile 0 into sA
  {
    // nothing to hide behind yet: results of the matrix unit may be read by the vector unit only some cycles
    // after the last pass
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
    mask_tile(0, sA);
    float mx[2] = {-INFINITY, -INFINITY};
#pragma unroll
    for (int n = 0; n < 8; ++n) max_slice(n, sA, mx);
    raise_reference(mx);
    kf_first = rm_frag(smem, 1, 0);
  }
  int stage = 0;
  for (int kb = 0; kb < nkb; ++kb) {
    const int next = stage == 2 ? 0 : stage + 1, after = next == 2 ? 0 : next + 1;
    step_scores(true, stage, 1, sA, sB, stage, 0);             // exponentials of tile 2 kb, scores of tile 2 kb + 1
    // block kb + 1 has landed (this wave's part; the barrier covers the rest; it was requested a whole block
    // ago) and nobody still reads the stage that block kb - 1 was in
    OPTSTAGE_BLOCK_SYNC();
    if (kb + 2 < nkb) issue_block(kb + 2, after);
    step_output(stage, 0, 2 * kb + 1, sA, sB, next, 0);
    step_scores(true, next, 0, sB, sA, stage, 1);              // exponentials of tile 2 kb + 1, scores of tile 2 kb + 2
    step_output(stage, 1, 2 * kb + 2, sB, sA, next, 1);
    stage = next;
  }
#undef OPTSTAGE_BLOCK_SYNC
#undef OPTSTAGE_MFMA_V
#undef OPTSTAGE_MFMA_A
  asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");

  float lt[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) lt[qt] = lsum[qt] + __shfl_xor(lsum[qt], 32, 64);
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    if (qglob[qt] >= seq) continue;
    const float inv = 1.f / lt[qt];
    bf16_t* orow = o + ((size_t)b * seq + qglob[qt]) * ldo + (size_t)a * D;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      OPTSTAGE_SB();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (bf16_t)(acc[qt][dt][4 * j + i] * inv);
        *reinterpret_cast<bf16x4_t*>(orow + 32 * dt + 8 * j + 4 * g) = r;
      }
    }
    if (g == 0) lse[((size_t)b * n_q + a) * seq + qglob[qt]] = mref[qt] * scale + logf(lt[qt]);
  }
#undef OPTSTAGE_SB
}


// ---- backward, dQ: grid (n_q, batch, ceil(seq / 256)); 4 waves (one per SIMD) -----------------------------
// Mirror image of the dK/dV kernel below.  Wave w owns queries q0 + 64 w .. + 63 as two 32-query tiles: their Q
// and dO operand fragments stay in registers (128) and dQ^T ([d 128][64 queries]) in accumulator registers, so
// every K / V fragment read from LDS feeds two MFMAs.  Key blocks of 64 (K and V rows) stream through a
// two-stage LDS ring loaded straight from global memory; one copy of the K tile serves S^T = K Q^T (16-byte row
// reads) and dQ^T += K^T dS^T (transposing reads), through the same chunk swizzle as in the dK/dV kernel.
// Also produces D_t = <dO_t, O_t> per query row and head (from the dO fragments it holds anyway) and stores it
// for the dK/dV kernel, which runs after this one.
constexpr int DQ_STAGE = 32768;              // K tile, V tile of 64 keys
constexpr int DQ_SMEM = 2 * DQ_STAGE;

__global__ __launch_bounds__(256) void attn_bwd_dq_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                        const bf16_t* __restrict__ dout, const float* __restrict__ lse,
                                                        float* __restrict__ delta, bf16_t* __restrict__ dqkv, int seq,
                                                        int n_q, int n_kv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqb = (seq + 255) / 256;
  const int q0 = (nqb - 1 - (int)blockIdx.z) * 256;          // longest rows are dispatched first, for every head
  const int a = blockIdx.x, b = blockIdx.y, kvh = a * n_kv / n_q;
  const int ld = (n_q + 2 * n_kv) * D, ldo = n_q * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const int wave_first_q = q0 + 64 * wave, wave_last_q = wave_first_q + 63;
  const float scale = rsqrtf((float)D), c = scale * LOG2E;

  // Q, dO operand fragments of this wave's queries (rows past the end are clamped: their results are not stored),
  // lse * log2(e) and D per query
  bf16x8_t Qf[2][8], dOf[2][8];
  float Lc[2], Dq[2];
  int qglob[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    qglob[qt] = wave_first_q + 32 * qt + c32;
    const int qrow = min(qglob[qt], seq - 1);
    const bf16_t* qp = base + (size_t)qrow * ld + (size_t)a * D + 8 * g;
    const bf16_t* dop = dout + ((size_t)b * seq + qrow) * ldo + (size_t)a * D + 8 * g;
    const bf16_t* op = o + ((size_t)b * seq + qrow) * ldo + (size_t)a * D + 8 * g;
    float dsum = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      Qf[qt][ks] = *reinterpret_cast<const bf16x8_t*>(qp + 16 * ks);
      dOf[qt][ks] = *reinterpret_cast<const bf16x8_t*>(dop + 16 * ks);
      const bf16x8_t of = *reinterpret_cast<const bf16x8_t*>(op + 16 * ks);
#pragma unroll
      for (int e = 0; e < 8; ++e) dsum = fmaf((float)dOf[qt][ks][e], (float)of[e], dsum);
    }
    Lc[qt] = -lse[((size_t)b * n_q + a) * seq + qrow] * LOG2E;
    Dq[qt] = dsum + __shfl_xor(dsum, 32, 64);                  // the two lanes of a row hold 64 columns each
    // stored negated: both backward kernels use -D as the initial value of their dP accumulators
    if (g == 0 && qglob[qt] < seq) delta[((size_t)b * n_q + a) * seq + qglob[qt]] = -Dq[qt];
  }
  // -D of this lane's two queries in every register of an accumulator-shaped tuple: the initial value of the dP^T
  // MFMAs, which then deliver dP^T - D
  f32x16_t negD[2];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int v = 0; v < 16; ++v) negD[qt][v] = -Dq[qt];
  // from here on the fragments are operands of MFMAs only: they move to the accumulation half of the register file
  // for good (the empty statements are where the move happens)
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" : "+a"(Qf[qt][ks]), "+a"(dOf[qt][ks]));
  f32x16_t acc[2][4];                          // [query tile][d tile]: lane = query, registers = d
#pragma unroll
  for (int qt = 0; qt < 2; ++qt)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][dt][v] = 0.f;

  int rm_addr[8];
  {
    const int f = ((c32 & 3) << 2) | ((c32 >> 2) & 3);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) rm_addr[ks] = c32 * 256 + (((2 * ks + g) ^ f) << 4);
  }
  int tr_addr[4][2];
  {
    const int cg = (lane >> 4) & 1, e = (lane >> 2) & 3, r = lane & 3;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int kq = 0; kq < 2; ++kq)
        tr_addr[dt][kq] = (4 * g + e) * 256 + (((4 * dt + 2 * cg + (r >> 1)) ^ (e << 2) ^ g ^ (kq << 1)) << 4) + (r & 1) * 8;
  }
  // tile loads: one instruction fills 4 rows (1 KB); wave w loads rows 16 w .. 16 w + 15 of the K and of the V tile
  unsigned voff[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = 16 * wave + 4 * j + (lane >> 4);
    const int chunk = (lane & 15) ^ (((lane >> 4) << 2) | j);
    voff[j] = (unsigned)row * (unsigned)ld * 2u + (unsigned)chunk * 16u;
  }
  auto make_desc = [](const void* p, unsigned bytes) {
    const unsigned long long ad = (unsigned long long)p;
    i32x4_t d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)ad);
    d[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(ad >> 32) & 0xffff);
    d[2] = (int)bytes;
    d[3] = 0x00020000;
    return d;
  };
  const i32x4_t rs = make_desc(base, (unsigned)seq * ld * 2u);
  const unsigned lds0 = (unsigned)(size_t)(lds_void_t*)smem;
  const unsigned k_off = (unsigned)(n_q + kvh) * D * 2u, v_off = (unsigned)(n_q + n_kv + kvh) * D * 2u;
  // All offsets go through the lane offset, which is what the range check sees: rows at or past seq read zero.
  auto issue_block = [&](int kb, int stage) {
    const unsigned rowoff = (unsigned)(64 * kb) * (unsigned)ld * 2u;
    const unsigned dst = lds0 + stage * DQ_STAGE + (16 * wave) * 256;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + j * 1024), "v"(voff[j] + rowoff + k_off), "s"(rs) : "memory", "m0");
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + 16384 + j * 1024), "v"(voff[j] + rowoff + v_off), "s"(rs) : "memory", "m0");
    }
  };
  typedef short i16x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
  auto tr_frag = [&](const char* tile, int dt, int t, int u) {
    const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u) * 256 + tr_addr[dt][0]));
    const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u + 8) * 256 + tr_addr[dt][1]));
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto rm_frag = [&](const char* tile, int t, int ks) {
    return *reinterpret_cast<const bf16x8_t*>(tile + t * 8192 + rm_addr[ks]);
  };

#define OPTSTAGE_SB() __builtin_amdgcn_sched_barrier(0)
  // the register-resident operands (Q, dO) sit in the accumulation half of the register file, next to dQ^T: an
  // MFMA takes its A / B operands from either half, and the vector half is left to the score tiles, the streaming
  // fragments and the addresses
#define OPTSTAGE_MFMA_V(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b))
#define OPTSTAGE_MFMA_0(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b))
  auto block = [&](int kb, int stage) {
    if (64 * kb > wave_last_q) return;                           // block above this wave's diagonal
    const char* sK = smem + stage * DQ_STAGE;
    const char* sV = sK + 16384;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int key0 = 64 * kb + 32 * t;
      if (key0 > wave_last_q) continue;                          // wave-uniform
      const bool edge = key0 + 31 > wave_first_q;                // touches the diagonal (keys past seq are masked by it)
      // lane = query, registers = keys key0 + 8 (v / 4) + 4 g + v % 4
      f32x16_t s[2], dp[2];
      bf16x8_t kf[2], vf[2];
      // ---- S^T = K Q^T (the first k-step starts from C = 0)
      kf[0] = rm_frag(sK, t, 0);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        OPTSTAGE_SB();
        if (ks < 7) kf[(ks + 1) & 1] = rm_frag(sK, t, ks + 1);
        else vf[0] = rm_frag(sV, t, 0);
        OPTSTAGE_SB();
        if (ks == 0) {
          OPTSTAGE_MFMA_0(s[0], kf[0], Qf[0][0]);
          OPTSTAGE_MFMA_0(s[1], kf[0], Qf[1][0]);
        } else {
          OPTSTAGE_MFMA_V(s[0], kf[ks & 1], Qf[0][ks]);
          OPTSTAGE_MFMA_V(s[1], kf[ks & 1], Qf[1][ks]);
        }
      }
      // ---- dP^T = V dO^T, with the exponentials of S^T under its MFMAs
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        OPTSTAGE_SB();
        if (ks < 7) vf[(ks + 1) & 1] = rm_frag(sV, t, ks + 1);
        OPTSTAGE_SB();
        if (ks == 0) {                                             // dP^T - D: the first k-step starts from C = -D
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(dp[0]) : "v"(vf[0]), "a"(dOf[0][0]), "v"(negD[0]));
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(dp[1]) : "v"(vf[0]), "a"(dOf[1][0]), "v"(negD[1]));
        } else {
          OPTSTAGE_MFMA_V(dp[0], vf[ks & 1], dOf[0][ks]);
          OPTSTAGE_MFMA_V(dp[1], vf[ks & 1], dOf[1][ks]);
        }
        OPTSTAGE_SB();
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int v = 2 * ks + e;
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) s[qt][v] = __builtin_amdgcn_exp2f(fmaf(s[qt][v], c, Lc[qt]));
        }
      }
      OPTSTAGE_SB();
      if (edge) {
        asm volatile("" ::: "memory");                             // a real branch: only diagonal tiles pay for the mask
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = key0 + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
          for (int qt = 0; qt < 2; ++qt)
            if (key > qglob[qt]) s[qt][v] = 0.f;
        }
      }
      // results of the matrix unit may be read by the vector unit only some cycles after the last pass
      asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
      OPTSTAGE_SB();
      // ---- dQ^T += K^T dS^T; dS^T = P^T (dP^T - D) of the second half runs under the MFMAs of the first (D is
      // already subtracted: it was the accumulator's initial value)
      bf16x8_t trf[2];
      trf[0] = tr_frag(sK, 0, t, 0);
#pragma unroll
      for (int v = 0; v < 8; ++v)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) dp[qt][v] = s[qt][v] * dp[qt][v];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8_t d0 = pack8(dp[0], u), d1 = pack8(dp[1], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const int n = u * 4 + dt;
          OPTSTAGE_SB();
          if (n < 7) trf[(n + 1) & 1] = tr_frag(sK, (dt + 1) & 3, t, dt == 3 ? 1 : u);
          OPTSTAGE_SB();
          acc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], d0, acc[0][dt], 0, 0, 0);
          acc[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], d1, acc[1][dt], 0, 0, 0);
          OPTSTAGE_SB();
          if (u == 0) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int v = 8 + 2 * dt + e;
#pragma unroll
              for (int qt = 0; qt < 2; ++qt) dp[qt][v] = s[qt][v] * dp[qt][v];
            }
          }
        }
      }
      OPTSTAGE_SB();
    }
  };
#undef OPTSTAGE_MFMA_V
#undef OPTSTAGE_MFMA_0
#undef OPTSTAGE_SB

  const int nkb = min((q0 + 255) / 64 + 1, (seq + 63) / 64);
  issue_block(0, 0);
  for (int kb = 0; kb < nkb; kb += 2) {
    // block kb has landed (this wave's part; the barrier covers the rest) and nobody still reads stage 1
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (kb + 1 < nkb) issue_block(kb + 1, 1);
    block(kb, 0);
    if (kb + 1 < nkb) {
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      if (kb + 2 < nkb) issue_block(kb + 2, 0);
      block(kb + 1, 1);
    }
  }

#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    if (qglob[qt] >= seq) continue;
    bf16_t* dq = dqkv + ((size_t)b * seq + qglob[qt]) * ld + (size_t)a * D;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4_t r;
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (bf16_t)(acc[qt][dt][4 * j + i] * scale);
        *reinterpret_cast<bf16x4_t*>(dq + 32 * dt + 8 * j + 4 * g) = r;
      }
  }
}

// ---- backward, dK / dV: grid (n_kv, batch, ceil(seq / 256)); 4 waves (one per SIMD) ----------------------
// Wave w owns keys k0 + 64 w .. + 63 as two 32-key tiles: their K operand fragments stay in registers for the
// whole kernel (the V rows of the workgroup's 256 keys stay in LDS: both operand sets do not fit beside the
// accumulators) and dK^T, dV^T ([d 128][64 keys] each) in the 256 accumulator registers, so every Q / dO
// fragment read from LDS feeds two MFMAs.  Query blocks of 64 (Q and dO rows plus their lse and D)
// stream through a two-stage LDS ring, loaded straight from global memory (`buffer_load ... lds`); one copy
// of a tile serves both contractions: over head_dim with 16-byte row reads (S = Q K^T, dP = dO V^T) and over
// the queries with transposing reads (dV^T += dO^T P, dK^T += Q^T dS).  16-byte chunk c of tile row r is
// stored at chunk c ^ f(r), f(r) = ((r & 3) << 2) | ((r >> 2) & 3): 16 consecutive rows get 16 different
// values (row reads of one chunk hit every bank once) and 4 consecutive rows differ in the 64-byte group
// (the 4 rows of a transposing read do too).
constexpr int DKV_STAGE = 32768 + 512;       // Q tile, dO tile, 64 lse, 64 D
constexpr int DKV_VTILE = 256 * 256;         // V rows of the workgroup's keys, behind the two stages
constexpr int DKV_SMEM = 2 * DKV_STAGE + DKV_VTILE;

// With grouped-query attention a kv head's gradient sums over n_q / n_kv query heads and the grid has only
// n_kv * batch * ceil(seq / 256) workgroups; `split` > 1 deals the query heads of a group to that many
// workgroups, each writing an fp32 partial ([part][batch][seq][kv head][K|V][128]) that attn_bwd_dkv_reduce sums
// in a fixed order.
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dout,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16_t* __restrict__ dqkv, float* __restrict__ partial, int split,
                                                         int seq, int n_q, int n_kv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k0 = blockIdx.z * 256;               // first key blocks (most queries) are dispatched first, for every head
  const int kvh = blockIdx.x / split, part = blockIdx.x % split, b = blockIdx.y;
  const int ld = (n_q + 2 * n_kv) * D, ldo = n_q * D;
  const bf16_t* base = qkv + (size_t)b * seq * ld;
  const int wave_first_k = k0 + 64 * wave;
  const float scale = rsqrtf((float)D), c = scale * LOG2E;

  // K, V operand fragments of this wave's keys (rows past the end are clamped: their results are not stored)
  bf16x8_t Kf[2][8];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int krow = min(wave_first_k + 32 * kk + c32, seq - 1);
    const bf16_t* kp = base + (size_t)krow * ld + (size_t)(n_q + kvh) * D + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) Kf[kk][ks] = *reinterpret_cast<const bf16x8_t*>(kp + 16 * ks);
  }
  f32x16_t accK[2][4], accV[2][4];            // [key tile][d tile]: lane = key, registers = d
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) { accK[kk][dt][v] = 0.f; accV[kk][dt][v] = 0.f; }

  // per-lane LDS addresses within a tile.  Row read of k-step ks: row c32 (+ 32 t), chunk 2 ks + g.
  int rm_addr[8];
  {
    const int f = ((c32 & 3) << 2) | ((c32 >> 2) & 3);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) rm_addr[ks] = c32 * 256 + (((2 * ks + g) ^ f) << 4);
  }
  // Transposing read (dt, kq): in each 16-lane group lane 4 e + r reads 8 bytes of row 4 g + e (+ 32 t + 16 u
  // + 8 kq), columns 32 dt + 16 cg + 4 r ..; f(row) = (e << 2) | (2 kq + g)
  int tr_addr[4][2];
  {
    const int cg = (lane >> 4) & 1, e = (lane >> 2) & 3, r = lane & 3;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int kq = 0; kq < 2; ++kq)
        tr_addr[dt][kq] = (4 * g + e) * 256 + (((4 * dt + 2 * cg + (r >> 1)) ^ (e << 2) ^ g ^ (kq << 1)) << 4) + (r & 1) * 8;
  }
  // tile loads: one instruction fills 4 rows (1 KB); wave w loads rows 16 w .. 16 w + 15 of Q and of dO.
  // Lane i: row 4 b + i / 16, stored chunk i % 16 = logical chunk ^ f(row), f = ((i / 16) << 2) | (b & 3).
  unsigned voff_q[4], voff_do[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = 16 * wave + 4 * j + (lane >> 4);
    const int chunk = (lane & 15) ^ (((lane >> 4) << 2) | j);
    voff_q[j] = (unsigned)row * (unsigned)ld * 2u + (unsigned)chunk * 16u;
    voff_do[j] = (unsigned)row * (unsigned)ldo * 2u + (unsigned)chunk * 16u;
  }
  auto make_desc = [](const void* p, unsigned bytes) {
    const unsigned long long a = (unsigned long long)p;
    i32x4_t d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    d[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)(a >> 32) & 0xffff);
    d[2] = (int)bytes;
    d[3] = 0x00020000;
    return d;
  };
  const i32x4_t rs_q = make_desc(base, (unsigned)seq * ld * 2u);
  const i32x4_t rs_do = make_desc(dout + (size_t)b * seq * ldo, (unsigned)seq * ldo * 2u);
  const i32x4_t rs_l = make_desc(lse + (size_t)b * n_q * seq, (unsigned)n_q * seq * 4u);
  const i32x4_t rs_d = make_desc(delta + (size_t)b * n_q * seq, (unsigned)n_q * seq * 4u);
  const unsigned lds0 = (unsigned)(size_t)(lds_void_t*)smem;

  // V rows of this wave's 64 keys -> LDS (16 loads of 4 rows), same layout as the streamed tiles
  const char* sV = smem + 2 * DKV_STAGE + wave * 16384;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int row = 4 * j + (lane >> 4);
    const int chunk = (lane & 15) ^ (((lane >> 4) << 2) | (j & 3));
    const unsigned vo = ((unsigned)(wave_first_k + row) * (unsigned)ld + (unsigned)(n_q + n_kv + kvh) * D) * 2u + (unsigned)chunk * 16u;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds0 + 2 * DKV_STAGE + wave * 16384 + j * 1024), "v"(vo), "s"(rs_q) : "memory", "m0");
  }
  const int rep = n_q / n_kv / split;                          // query heads of the group handled here
  const int qb0 = k0 / 64, nqb = (seq + 63) / 64 - qb0;       // query blocks at or after the first key
  const int iters = rep * nqb;
  // All offsets go through the lane offset, which is what the range check sees: rows at or past seq read zero.
  auto issue_block = [&](int it, int stage) {
    const int a = (kvh * split + part) * rep + it / nqb;
    const int r0 = 64 * (qb0 + it % nqb);
    const unsigned oq = ((unsigned)r0 * (unsigned)ld + (unsigned)a * D) * 2u;
    const unsigned od = ((unsigned)r0 * (unsigned)ldo + (unsigned)a * D) * 2u;
    const unsigned dst = lds0 + stage * DKV_STAGE + (16 * wave) * 256;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + j * 1024), "v"(voff_q[j] + oq), "s"(rs_q) : "memory", "m0");
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst + 16384 + j * 1024), "v"(voff_do[j] + od), "s"(rs_do) : "memory", "m0");
    }
    if (wave < 2) {                            // wave 0: lse of the 64 queries, wave 1: D
      const unsigned vo = ((unsigned)a * (unsigned)seq + (unsigned)min(r0 + lane, seq - 1)) * 4u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                   :: "s"(lds0 + stage * DKV_STAGE + 32768 + wave * 256), "v"(vo), "s"(wave == 0 ? rs_l : rs_d) : "memory", "m0");
    }
  };
  typedef short i16x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
  auto tr_frag = [&](const char* tile, int dt, int t, int u) {
    const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u) * 256 + tr_addr[dt][0]));
    const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(tile + (32 * t + 16 * u + 8) * 256 + tr_addr[dt][1]));
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto rm_frag = [&](const char* tile, int t, int ks) {
    return *reinterpret_cast<const bf16x8_t*>(tile + t * 8192 + rm_addr[ks]);
  };

#define OPTSTAGE_SB() __builtin_amdgcn_sched_barrier(0)
  // VGPR-result MFMA in assembly: the compiler would place the score tiles in accumulator registers, all 256
  // of which hold dK, dV.  Readers of the result keep >= 2 MFMAs (or an s_nop) behind the last write.
#define OPTSTAGE_MFMA_V(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
#define OPTSTAGE_MFMA_0(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b))
  auto block = [&](int it, int stage) {
    const int r0 = 64 * (qb0 + it % nqb);
    if (r0 + 63 < wave_first_k) return;                          // all queries precede this wave's keys
    const char* sQ = smem + stage * DKV_STAGE;
    const char* sDO = sQ + 16384;
    const float* sL = reinterpret_cast<const float*>(sQ + 32768);
    const float* sD = sL + 64;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int q0 = r0 + 32 * t;
      if (q0 + 31 < wave_first_k) continue;                      // wave-uniform
      const bool edge = q0 < wave_first_k + 63 || q0 + 32 > seq;   // touches the diagonal or the ragged tail
      // lane = key, registers = queries q0 + 8 (v / 4) + 4 g + v % 4
      f32x16_t s[2], dp[2];
      f32x4_t nL[4];                                               // -lse * log2(e) of this lane's queries
      f32x16_t negD;                                               // -D of this lane's queries, in accumulator order
      bf16x8_t qf[2], df[2], vf[2][2];
      // ---- S = Q K^T: fragment of k-step ks + 1 requested before the MFMAs of k-step ks
      qf[0] = rm_frag(sQ, t, 0);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        OPTSTAGE_SB();
        if (ks < 7) {
          qf[(ks + 1) & 1] = rm_frag(sQ, t, ks + 1);
        } else {
          df[0] = rm_frag(sDO, t, 0);
          vf[0][0] = rm_frag(sV, 0, 0);
          vf[0][1] = rm_frag(sV, 1, 0);
        }
        if (ks < 4) nL[ks] = *reinterpret_cast<const f32x4_t*>(sL + 32 * t + 8 * ks + 4 * g);
        else {
          const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(sD + 32 * t + 8 * (ks - 4) + 4 * g);
#pragma unroll
          for (int i = 0; i < 4; ++i) negD[4 * (ks - 4) + i] = d4[i];
        }
        OPTSTAGE_SB();
        if (ks == 0) {                                             // the first k-step starts from C = 0
          OPTSTAGE_MFMA_0(s[0], qf[0], Kf[0][0]);
          OPTSTAGE_MFMA_0(s[1], qf[0], Kf[1][0]);
        } else {
          OPTSTAGE_MFMA_V(s[0], qf[ks & 1], Kf[0][ks]);
          OPTSTAGE_MFMA_V(s[1], qf[ks & 1], Kf[1][ks]);
        }
        OPTSTAGE_SB();
        if (ks >= 4) {
#pragma unroll
          for (int i = 0; i < 4; ++i) nL[ks - 4][i] *= -LOG2E;
        }
      }
      // ---- dP = dO V^T, with the exponentials of S (2 registers x 2 key tiles per k-step) under its MFMAs
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        OPTSTAGE_SB();
        if (ks < 7) {
          df[(ks + 1) & 1] = rm_frag(sDO, t, ks + 1);
          vf[(ks + 1) & 1][0] = rm_frag(sV, 0, ks + 1);
          vf[(ks + 1) & 1][1] = rm_frag(sV, 1, ks + 1);
        }
        OPTSTAGE_SB();
        if (ks == 0) {                                             // dP - D: the first k-step starts from C = -D
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(dp[0]) : "v"(df[0]), "v"(vf[0][0]), "v"(negD));
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(dp[1]) : "v"(df[0]), "v"(vf[0][1]), "v"(negD));
        } else {
          OPTSTAGE_MFMA_V(dp[0], df[ks & 1], vf[ks & 1][0]);
          OPTSTAGE_MFMA_V(dp[1], df[ks & 1], vf[ks & 1][1]);
        }
        OPTSTAGE_SB();
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int v = 2 * ks + e;
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) s[kk][v] = __builtin_amdgcn_exp2f(fmaf(s[kk][v], c, nL[v >> 2][v & 3]));
        }
      }
      OPTSTAGE_SB();
      if (edge) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int qg = q0 + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
          for (int kk = 0; kk < 2; ++kk)
            if (qg < wave_first_k + 32 * kk + c32 || qg >= seq) s[kk][v] = 0.f;
        }
      }
      OPTSTAGE_SB();
      // ---- dV^T += dO^T P, with dS = P (dP - D) under its MFMAs (the first two MFMAs cover the dP latency)
      bf16x8_t trf[2];
      trf[0] = tr_frag(sDO, 0, t, 0);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8_t p0 = pack8(s[0], u), p1 = pack8(s[1], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const int n = u * 4 + dt;
          OPTSTAGE_SB();
          if (n < 7) trf[(n + 1) & 1] = tr_frag(sDO, (dt + 1) & 3, t, dt == 3 ? 1 : u);
          else trf[0] = tr_frag(sQ, 0, t, 0);
          OPTSTAGE_SB();
          accV[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], p0, accV[0][dt], 0, 0, 0);
          accV[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], p1, accV[1][dt], 0, 0, 0);
          OPTSTAGE_SB();
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int v = 2 * n + e;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) dp[kk][v] = s[kk][v] * dp[kk][v];
          }
        }
      }
      // ---- dK^T += Q^T dS
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8_t d0 = pack8(dp[0], u), d1 = pack8(dp[1], u);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const int n = u * 4 + dt;
          OPTSTAGE_SB();
          if (n < 7) trf[(n + 1) & 1] = tr_frag(sQ, (dt + 1) & 3, t, dt == 3 ? 1 : u);
          OPTSTAGE_SB();
          accK[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], d0, accK[0][dt], 0, 0, 0);
          accK[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trf[n & 1], d1, accK[1][dt], 0, 0, 0);
        }
      }
      OPTSTAGE_SB();
    }
  };
#undef OPTSTAGE_MFMA_V
#undef OPTSTAGE_MFMA_0
#undef OPTSTAGE_SB

  if (iters > 0) issue_block(0, 0);
  for (int it = 0; it < iters; it += 2) {
    // block `it` has landed (this wave's part; the barrier covers the rest) and nobody still reads stage 1
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (it + 1 < iters) issue_block(it + 1, 1);
    block(it, 0);
    if (it + 1 < iters) {
      asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
      if (it + 2 < iters) issue_block(it + 2, 0);
      block(it + 1, 1);
    }
  }

#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int kglob = wave_first_k + 32 * kk + c32;
    if (kglob >= seq) continue;
    if (split > 1) {
      float* prow = partial + ((((size_t)part * gridDim.y + b) * seq + kglob) * n_kv + kvh) * 2 * D;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          f32x4_t rk, rv;
#pragma unroll
          for (int i = 0; i < 4; ++i) { rk[i] = accK[kk][dt][4 * j + i]; rv[i] = accV[kk][dt][4 * j + i]; }
          *reinterpret_cast<f32x4_t*>(prow + 32 * dt + 8 * j + 4 * g) = rk;
          *reinterpret_cast<f32x4_t*>(prow + D + 32 * dt + 8 * j + 4 * g) = rv;
        }
      continue;
    }
    bf16_t* krow = dqkv + ((size_t)b * seq + kglob) * ld + (size_t)(n_q + kvh) * D;
    bf16_t* vrow = dqkv + ((size_t)b * seq + kglob) * ld + (size_t)(n_q + n_kv + kvh) * D;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x4_t rk, rv;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          rk[i] = (bf16_t)(accK[kk][dt][4 * j + i] * scale);
          rv[i] = (bf16_t)accV[kk][dt][4 * j + i];
        }
        *reinterpret_cast<bf16x4_t*>(krow + 32 * dt + 8 * j + 4 * g) = rk;
        *reinterpret_cast<bf16x4_t*>(vrow + 32 * dt + 8 * j + 4 * g) = rv;
      }
  }
}

// sums the `split` partials of dK, dV (fixed order), scales dK by 1 / sqrt(d) and stores bf16 into the packed
// gradient rows: one thread per 4 columns of one (token, kv head, K|V)
__global__ void attn_bwd_dkv_reduce(const float* __restrict__ partial, bf16_t* __restrict__ dqkv, int split, int rows,
                                    int n_q, int n_kv) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t per_part = (size_t)rows * n_kv * 2 * D;
  if (idx * 4 >= per_part) return;
  const size_t e = idx * 4;
  const int col = (int)(e % D);
  const int kv = (int)((e / D) % 2);
  const int h = (int)((e / (2 * D)) % n_kv);
  const size_t row = e / ((size_t)2 * D * n_kv);
  f32x4_t acc = *reinterpret_cast<const f32x4_t*>(partial + e);
  for (int p = 1; p < split; ++p) {
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(partial + p * per_part + e);
    acc[0] += v[0]; acc[1] += v[1]; acc[2] += v[2]; acc[3] += v[3];
  }
  const float sc = kv == 0 ? rsqrtf((float)D) : 1.f;
  bf16x4_t o;
  o[0] = (bf16_t)(acc[0] * sc); o[1] = (bf16_t)(acc[1] * sc); o[2] = (bf16_t)(acc[2] * sc); o[3] = (bf16_t)(acc[3] * sc);
  const int ld = (n_q + 2 * n_kv) * D;
  *reinterpret_cast<bf16x4_t*>(dqkv + row * ld + (size_t)(n_q + kv * n_kv + h) * D + col) = o;
}

}  // namespace

// how many workgroups share the query heads of one kv head in the dK/dV kernel: enough to give every compute
// unit about two workgroups, a divisor of n_q / n_kv
int attn_dkv_split(int seq, int batch, int n_q, int n_kv) {
  const int rep = n_q / n_kv;
  const long wgs = (long)n_kv * batch * ((seq + 255) / 256);
  int split = 1;
  while (split < rep && wgs * split < 448 && rep % (split * 2) == 0) split *= 2;
  return split;
}

// bf16, head_dim 128, and per-sequence tensors addressable with 32-bit byte offsets (buffer loads)
bool attn_mfma_applies(int dtype, int d, int seq, int n_q, int n_kv) {
  return dtype == DT_BF16 && d == 128 && (unsigned long long)(seq + 256) * (n_q + 2 * n_kv) * 128 * 2 < 0xF0000000ull;
}

hipError_t launch_attn_fwd_mfma(const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv, hipStream_t s) {
  static LdsAttrOnce lds_attr;
  if (hipError_t e = lds_attr.ensure(reinterpret_cast<const void*>(attn_fwd_mfma), FWD_SMEM); e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_fwd_mfma, dim3(n_q, batch, (seq + 255) / 256), dim3(256), FWD_SMEM, s, (const bf16_t*)qkv, (bf16_t*)o, lse, seq, n_q, n_kv);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv, float* ws,
                                int seq, int batch, int n_q, int n_kv, hipStream_t s) {
  hipError_t e;
  static LdsAttrOnce dq_attr, dkv_attr;
  if ((e = dq_attr.ensure(reinterpret_cast<const void*>(attn_bwd_dq_mfma), DQ_SMEM)) != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_mfma, dim3(n_q, batch, (seq + 255) / 256), dim3(256), DQ_SMEM, s, (const bf16_t*)qkv,
      (const bf16_t*)o, (const bf16_t*)dout, lse, ws, (bf16_t*)dqkv, seq, n_q, n_kv);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if ((e = dkv_attr.ensure(reinterpret_cast<const void*>(attn_bwd_dkv_mfma), DKV_SMEM)) != hipSuccess) return e;
  const int split = attn_dkv_split(seq, batch, n_q, n_kv);
  float* partial = ws + (size_t)batch * n_q * seq;            // behind the D array
  hipLaunchKernelGGL(attn_bwd_dkv_mfma, dim3(n_kv * split, batch, (seq + 255) / 256), dim3(256), DKV_SMEM, s,
      (const bf16_t*)qkv, (const bf16_t*)dout, lse, ws, (bf16_t*)dqkv, partial, split, seq, n_q, n_kv);
  if (split > 1) {
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t quads = (size_t)batch * seq * n_kv * 2 * D / 4;
    hipLaunchKernelGGL(attn_bwd_dkv_reduce, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, partial, (bf16_t*)dqkv,
        split, batch * seq, n_q, n_kv);
  }
  return hipGetLastError();
}
