// bf16 MFMA GEMM for gfx950: C[M,N] = sum_k A(m,k) * B(n,k), fp32 accumulation.
//
// These are the three linear maps of a stage (paper Sec. 2.2): forward Y = X W^T (NT), backward for
// activations dX = dY W (NT against the transposed weight copy), backward for weights dW += dY^T X (TN).
//
// Design (CDNA4): one workgroup of 4 or 8 waves owns a BM x BN output tile (256 x 256 for large problems);
// the K loop advances 64 elements at a time through LDS tiles (two buffers in the register-staged kernel, a ring
// of five operand slots in the direct kernels) with one barrier per step.
// Large problems with K % 64 == 0 load their tiles straight from global memory into LDS (no registers, no
// ds_write; see the direct kernels below); everything else stages tiles global -> registers -> LDS.  LDS tiles
// are always [row][64 k] with the 16-byte chunk index XOR-swizzled by the row so that both the 16-byte operand reads
// of v_mfma_f32_32x32x16_bf16 and the tile writes are bank-conflict
// free.  Operands that are contiguous along their output index (TN) are transposed in registers on the
// way into LDS (each thread gathers a KV x 8 patch and writes 8 k-contiguous pieces), so the MFMA read
// path is identical for every layout.  The MFMA is issued with the B fragment as its first operand:
// each lane then owns 4 consecutive n of one m, which gives 8-byte (bf16) / 16-byte (fp32) row-major
// global accesses in the epilogue.  Workgroup ids are remapped so that the tiles resident on one XCD
// (ids congruent mod 8) form a compact patch of the output and share A/B panels in that XCD's L2.
#include <utility>

#include "common.h"

namespace {

constexpr int BK = 64;           // k elements per LDS tile
constexpr int ROW_BYTES = 128;   // 64 bf16

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// ---- global -> register staging -------------------------------------------------------------------
// K-contiguous operand: element (r, k) at p[r * ld + k].  Thread handles R_T/32 16-byte chunks.
template <int R_T, int NTH> struct StageKC {
  static constexpr int NCH = R_T * 8 / NTH;
  uint4 reg[NCH];
  __device__ __forceinline__ void load(const bf16_t* p, int ld, int row0, int rows, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int q = tid + NTH * i;
      int row = q >> 3, c = q & 7;
      int gr = row0 + row, gk = k0 + c * 8;
      if (gr < rows && gk < K)
        reg[i] = *reinterpret_cast<const uint4*>(p + (size_t)gr * ld + gk);
      else
        reg[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int q = tid + NTH * i;
      int row = q >> 3, c = q & 7;
      *reinterpret_cast<uint4*>(lds + row * ROW_BYTES + ((c ^ swz(row)) << 4)) = reg[i];
    }
  }
};

// Row-contiguous operand: element (r, k) at p[k * ld + r].  Thread gathers KV k-rows x 8 r and writes
// 8 pieces of KV k-contiguous elements.
template <int R_T, int NTH> struct StageRC {
  static constexpr int KV = R_T * 8 / NTH;   // k-rows per thread: 8 (16-byte LDS stores) or 4 (8-byte stores)
  static_assert(KV == 8 || KV == 4, "unsupported tile / thread-count combination");
  uint4 reg[KV];
  __device__ __forceinline__ static void coords(int tid, int& rc, int& kg) {
    if (KV == 8) {          // R_T / 8 row chunks x 8 k-groups; 8 consecutive lanes hit 8 distinct 16-byte chunks
      rc = tid % (R_T / 8);
      kg = tid / (R_T / 8);
    } else {                // 8-byte stores: lanes 0-7 vary the row chunk, lane bit 3 the half of the 16-byte chunk
      const int hi = tid >> 4;
      rc = (tid & 7) | ((hi % (R_T / 64)) << 3);
      kg = ((tid >> 3) & 1) | ((hi / (R_T / 64)) << 1);
    }
  }
  __device__ __forceinline__ void load(const bf16_t* p, int ld, int row0, int rows, int k0, int K, int tid) {
    int rc, kg;
    coords(tid, rc, kg);
    int gr = row0 + rc * 8;
#pragma unroll
    for (int kk = 0; kk < KV; ++kk) {
      int gk = k0 + kg * KV + kk;
      if (gr < rows && gk < K)
        reg[kk] = *reinterpret_cast<const uint4*>(p + (size_t)gk * ld + gr);
      else
        reg[kk] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(char* lds, int tid) const {
    int rc, kg;
    coords(tid, rc, kg);
    const uint32_t* w = reinterpret_cast<const uint32_t*>(reg);   // w[kk*4 + i/2] holds elements i, i+1 of k-row kk
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t out[KV / 2];
#pragma unroll
      for (int pr = 0; pr < KV / 2; ++pr) {
        uint32_t a = w[(2 * pr) * 4 + (i >> 1)], b = w[(2 * pr + 1) * 4 + (i >> 1)];
        out[pr] = (i & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
      }
      int row = rc * 8 + i;
      int koff = kg * KV;
      char* dst = lds + row * ROW_BYTES + ((((koff >> 3)) ^ swz(row)) << 4) + (koff & 7) * 2;
      if (KV == 8)
        *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2 % (KV / 2)], out[3 % (KV / 2)]);
      else
        *reinterpret_cast<uint2*>(dst) = make_uint2(out[0], out[1]);
    }
  }
};

template <int R_T, int NTH, bool RC> struct StageSel { typedef StageKC<R_T, NTH> type; };
template <int R_T, int NTH> struct StageSel<R_T, NTH, true> { typedef StageRC<R_T, NTH> type; };

// Epilogue through LDS for 256 x 256 workgroup tiles: each wave transposes its accumulator tile (32 TM rows
// x 128 columns), 32 * 128 KB / (NWAVES * 16 KB) rows at a time, through a private slice of the 128 KB of
// LDS (16-byte chunks XOR-swizzled by the row, conflict free both ways), so that global memory sees whole
// 512-byte row segments instead of 16-byte pieces of 32 different rows.  The caller has made sure that no
// wave still reads operand tiles.
template <int EPI, int TM, int TN, int NWAVES>
__device__ __forceinline__ void epilogue_via_lds(f32x16_t (&acc)[TM][TN], char* smem, int wave, int lane, void* Cv,
                                                 const bf16_t* R, int M, int N, int ldc, int mw, int nw) {
  static_assert(TN == 4, "a wave tile is 128 columns wide");
  constexpr int SLICE = 131072 / NWAVES, IPP = SLICE / 16384;     // MFMA tile rows (32 matrix rows) per pass
  static_assert(IPP >= 1 && TM % IPP == 0, "wave tile must split into whole passes");
  constexpr int NIT = 16 * IPP;                                   // row pairs per pass
  char* const wl = smem + wave * SLICE;
  const int khalf = lane >> 5;
  const int c = lane & 31;
  const int n = nw + c * 4;
#pragma unroll
  for (int pass = 0; pass < TM / IPP; ++pass) {
    // accumulate / residual: request this pass's rows of the old values first, so that their latency runs
    // under the LDS transposition
    // (only where the register budget allows it: 4-wave kernels)
    constexpr bool PRE = NWAVES == 4;
    f32x4_t cold[EPI == EPI_ACCUM && PRE ? NIT : 1];
    bf16x4_t rold[EPI == EPI_RESID && PRE ? NIT : 1];
    if ((EPI == EPI_ACCUM || EPI == EPI_RESID) && PRE) {
#pragma unroll
      for (int p2 = 0; p2 < NIT; ++p2) {
        const int m = mw + pass * IPP * 32 + 2 * p2 + khalf;
        const bool ok = m < M && n < N;
        const size_t off = (size_t)m * ldc + n;
        if (EPI == EPI_ACCUM) {
          f32x4_t z = {0.f, 0.f, 0.f, 0.f};
          cold[p2] = ok ? __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(Cv) + off)) : z;
        } else {
          bf16x4_t z = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
          rold[p2] = ok ? *reinterpret_cast<const bf16x4_t*>(R + off) : z;
        }
      }
    }
#pragma unroll
    for (int i2 = 0; i2 < IPP; ++i2) {
      const int row = i2 * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int chunk = j * 8 + g * 2 + khalf;
          f32x4_t v;
          v[0] = acc[pass * IPP + i2][j][g * 4 + 0]; v[1] = acc[pass * IPP + i2][j][g * 4 + 1];
          v[2] = acc[pass * IPP + i2][j][g * 4 + 2]; v[3] = acc[pass * IPP + i2][j][g * 4 + 3];
          *reinterpret_cast<f32x4_t*>(wl + row * 512 + ((chunk ^ (row & 31)) << 4)) = v;
        }
    }
#pragma unroll
    for (int p2 = 0; p2 < NIT; ++p2) {
      const int row = 2 * p2 + khalf;
      const int m = mw + pass * IPP * 32 + row;
      f32x4_t v = *reinterpret_cast<const f32x4_t*>(wl + row * 512 + ((c ^ (row & 31)) << 4));
      if (m < M && n < N) {
        const size_t off = (size_t)m * ldc + n;
        if (EPI == EPI_STOREF) {
          __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(Cv) + off));
        } else if (EPI == EPI_ACCUM) {
          const f32x4_t o = PRE ? cold[PRE ? p2 : 0] : *reinterpret_cast<const f32x4_t*>(reinterpret_cast<const float*>(Cv) + off);
          v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
          __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(Cv) + off));
        } else {
          if (EPI == EPI_RESID) {
            const bf16x4_t r = PRE ? rold[PRE ? p2 : 0] : *reinterpret_cast<const bf16x4_t*>(R + off);
            v[0] += (float)r[0]; v[1] += (float)r[1]; v[2] += (float)r[2]; v[3] += (float)r[3];
          }
          bf16x4_t o;
          o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
          *reinterpret_cast<bf16x4_t*>(reinterpret_cast<bf16_t*>(Cv) + off) = o;
        }
      }
    }
  }
}

// ---- kernel ---------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool A_RC, bool B_RC, int EPI>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                        void* __restrict__ Cv, const bf16_t* __restrict__ R, int M,
                                                        int N, int K, int lda, int ldb, int ldc, int tiles_m,
                                                        int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, BUF = A_BYTES + B_BYTES;
  constexpr int NTH = 64 * WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave in m and n

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // XCD-aware tile order: consecutive hardware ids go to different XCDs, so give every XCD one
  // contiguous range of the tile sequence, and walk that sequence in groups of 8 tile rows.
  int pid = blockIdx.x;
  const int nblk = tiles_m * tiles_n;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  constexpr int GM = 8;
  const int grp = pid / (GM * tiles_n);
  const int first_m = grp * GM;
  const int gsz = min(tiles_m - first_m, GM);
  const int in_grp = pid - grp * GM * tiles_n;
  const int tile_m = first_m + in_grp % gsz, tile_n = in_grp / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  typename StageSel<BM, NTH, A_RC>::type sa;
  typename StageSel<BN, NTH, B_RC>::type sb;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // per-lane LDS read offsets (row part); the k chunk is added per k-step
  int a_off[TM], a_sw[TM], b_off[TN], b_sw[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    int row = wm * (BM / WM) + i * 32 + (lane & 31);
    a_off[i] = row * ROW_BYTES;
    a_sw[i] = swz(row);
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    int row = wn * (BN / WN) + j * 32 + (lane & 31);
    b_off[j] = A_BYTES + row * ROW_BYTES;
    b_sw[j] = swz(row);
  }
  const int khalf = lane >> 5;

  const int nk = (K + BK - 1) / BK;
  char* const buf0 = smem;
  char* const buf1 = smem + BUF;

  // operand fragments of one 16-wide k-step
  auto load_frags = [&](bf16x8_t (&af)[TM], bf16x8_t (&bfr)[TN], const char* buf, int ks) {
    const int chunk = ks * 2 + khalf;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(buf + a_off[i] + ((chunk ^ a_sw[i]) << 4));
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(buf + b_off[j] + ((chunk ^ b_sw[j]) << 4));
  };
  auto mma = [&](const bf16x8_t (&af)[TM], const bf16x8_t (&bfr)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
  };

  // Software pipeline.  LDS holds tiles kt (cur) and kt+1 (nxt); registers hold tile kt+2 in flight.
  // Fragments are double-buffered so the LDS reads of k-step ks+1 run under the MFMAs of k-step ks, and
  // the one barrier per tile sits before the last k-step, with a full k-step of MFMAs already queued;
  // after it the freed cur buffer takes tile kt+2 and the first fragments of tile kt+1 are fetched.
  sa.load(A, lda, m0, M, 0, K, tid);
  sb.load(B, ldb, n0, N, 0, K, tid);
  sa.store(buf0, tid);
  sb.store(buf0 + A_BYTES, tid);
  sa.load(A, lda, m0, M, BK, K, tid);
  sb.load(B, ldb, n0, N, BK, K, tid);
  sa.store(buf1, tid);
  sb.store(buf1 + A_BYTES, tid);
  __syncthreads();

  bf16x8_t fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  load_frags(fa0, fb0, buf0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = (kt & 1) ? buf1 : buf0;
    char* nxt = (kt & 1) ? buf0 : buf1;
    sa.load(A, lda, m0, M, (kt + 2) * BK, K, tid);
    sb.load(B, ldb, n0, N, (kt + 2) * BK, K, tid);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(fa1, fb1, cur, 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(fa0, fb0, cur, 2);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(fa1, fb1, cur, 3);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    // every wave has issued its last read of cur and its writes of nxt: wait for LDS traffic only
    // (global loads of tile kt+2 stay in flight), then meet
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    load_frags(fa0, fb0, nxt, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    sa.store(cur, tid);
    sb.store(cur + A_BYTES, tid);
  }

  if constexpr (BM == 256 && BN == 256 && TN == 4) {
    __syncthreads();                                 // every wave is done with the operand tiles
    epilogue_via_lds<EPI, TM, TN, WM * WN>(acc, smem, wave, lane, Cv, R, M, N, ldc, m0 + wm * (BM / WM), n0 + wn * (BN / WN));
    return;
  }
  // epilogue: lane owns m = .. + (lane & 31) and, per register group g, n = .. + 8 g + 4 (lane >> 5) + 0..3
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * (BM / WM) + i * 32 + (lane & 31);
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * (BN / WN) + j * 32 + g * 8 + khalf * 4;
        if (n >= N) continue;
        const size_t off = (size_t)m * ldc + n;
        float v0 = acc[i][j][g * 4 + 0], v1 = acc[i][j][g * 4 + 1], v2 = acc[i][j][g * 4 + 2], v3 = acc[i][j][g * 4 + 3];
        if (EPI == EPI_STOREF) {
          f32x4_t c = {v0, v1, v2, v3};
          *reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(Cv) + off) = c;
        } else if (EPI == EPI_ACCUM) {
          float* C = reinterpret_cast<float*>(Cv);
          f32x4_t c = *reinterpret_cast<const f32x4_t*>(C + off);
          c[0] += v0; c[1] += v1; c[2] += v2; c[3] += v3;
          *reinterpret_cast<f32x4_t*>(C + off) = c;
        } else {
          if (EPI == EPI_RESID) {
            bf16x4_t r = *reinterpret_cast<const bf16x4_t*>(R + off);
            v0 += (float)r[0]; v1 += (float)r[1]; v2 += (float)r[2]; v3 += (float)r[3];
          }
          bf16x4_t o;
          o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
          *reinterpret_cast<bf16x4_t*>(reinterpret_cast<bf16_t*>(Cv) + off) = o;
        }
      }
    }
  }
}

// ---- kernels with direct global -> LDS tile loads (NT and TN) -----------------------------------------
// 256 x 256 x 64 tiles, 2 x 2 waves (one per SIMD; each owns 128 x 128 of the output in 256 accumulator
// registers).  The tiles never pass through registers: every wave issues 16 `buffer_load_dwordx4 ... lds` per
// k-tile, each filling 1 KB of LDS (lane i writes 16 bytes at base + 16 i); which global address a lane loads
// realises the LDS swizzle.  Requires K % 64 == 0 and operands below 4 GiB (checked on the host); rows or
// columns past the operand read as zero through the buffer range check.
//
//  NT (operands contiguous along k): a stage holds [256 rows][64 k]; the load for rows 8 q .. 8 q + 7 has lane i
//     fetch row 8 q + i / 8, logical 16-byte chunk (i % 8) ^ swz(row); fragments are plain 16-byte reads.
//  TN (operands contiguous along their output index): a stage holds the tile as it lies in memory,
//     [64 k][256 columns]; one load fills k-rows 2 b, 2 b + 1, lane i fetching k-row 2 b + i / 32, logical chunk
//     (i % 32) ^ ((k & 3) << 2).  Fragments come from the transposing read ds_read_b64_tr_b16: in every 16-lane
//     group lane 4 e + r reads 8 bytes of k-row e, columns 4 r .. 4 r + 3, and the instruction hands lane i the
//     4 k values of column i; two of them make the 8 k of an MFMA operand.  The chunk XOR spreads the 4 k-rows
//     of such a read over the four 64-byte bank groups.
//
// With a single wave per SIMD nothing hides an instruction that waits, so the main loop is laid out by hand
// (the scheduling barriers pin the order):
//  * LDS is a ring of five 32 KB slots that the operand tiles take in the order A0 B0 A1 B1 A2 ...; a tile's
//    operands may lie in any two of them, so the per-lane fragment addresses are rebuilt (one add each) for
//    the next tile under MFMAs that have nothing else to issue; for TN the k-step is an immediate offset.
//  * Fragment reads are issued ahead of every pair of MFMAs (k-step s + 1 is fetched under the MFMAs of
//    k-step s); the fragments of the last k-step of a tile are requested early in the k-step before, so they
//    have landed when the tile barrier is reached.
//  * The loop is rotated so that the one barrier per tile (next tile landed, two slots free to refill) sits at
//    the top of the trip; it waits for all of this wave's loads but the newest eight, which belong to the tile
//    after the next one.
//  * One tile load goes out ahead of every fourth MFMA.  Issued back to back (16 loads by each of four waves at
//    the same point of the loop) they fill the address queue of the texture unit, which blocks the waves that
//    issue them and the MFMAs behind; the uneven request stream also cost a third more L2 misses.
//  * A tile index past the end is fetched through a zero-length descriptor, which zero-fills its slot, so the
//    number of loads in flight is the same on every trip and the waits need no second code path.
//  * The tile loads are written in assembly: issued through the compiler builtin, every later transposing
//    read is ordered after them with a full vmcnt(0) wait, which serialises the loop.  The one wait + barrier
//    per tile orders them instead.
typedef __attribute__((address_space(3))) void lds_void_t;
typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
typedef int i32x4_t __attribute__((ext_vector_type(4)));

// Epilogue of the direct kernels for bf16 outputs: the wave converts its 128 x 128 accumulator tile to bf16
// (after adding the residual, read in accumulator layout, when there is one), transposes it through its own
// 32 KB of LDS ([128 rows][256 B], 16-byte chunks XOR-swizzled by the row) and writes whole 256-byte row
// segments, 16 bytes per lane.  Rows 16..31 of every 32 keep the two 8-byte halves of a chunk swapped so that
// a 32-lane 8-byte write touches all 64 banks once.
template <int EPI>
__device__ __forceinline__ void epilogue_bf16_rows(f32x16_t (&acc)[4][4], char* smem, int wave, int lane, bf16_t* C,
                                                   const bf16_t* R, int M, int N, int ldc, int mw, int nw) {
  char* const wl = smem + wave * 32768;
  const int khalf = lane >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = i * 32 + (lane & 31);
    const int hoff = ((khalf ^ ((row >> 4) & 1)) << 3);
    bf16x4_t res[16];
    if (EPI == EPI_RESID) {
      const int m = mw + row;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = nw + j * 32 + g * 8 + khalf * 4;
          bf16x4_t r = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
          if (m < M && n < N) r = *reinterpret_cast<const bf16x4_t*>(R + (size_t)m * ldc + n);
          res[j * 4 + g] = r;
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float v0 = acc[i][j][g * 4 + 0], v1 = acc[i][j][g * 4 + 1], v2 = acc[i][j][g * 4 + 2], v3 = acc[i][j][g * 4 + 3];
        if (EPI == EPI_RESID) {
          const bf16x4_t r = res[j * 4 + g];
          v0 += (float)r[0]; v1 += (float)r[1]; v2 += (float)r[2]; v3 += (float)r[3];
        }
        bf16x4_t o;
        o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
        const int chunk = j * 4 + g;
        *reinterpret_cast<bf16x4_t*>(wl + row * 256 + ((chunk ^ (row & 15)) << 4) + hoff) = o;
      }
  }
  // every wave reads back only what it wrote itself: no workgroup barrier
  const int c = lane & 15, rsub = lane >> 4;
  const int n = nw + c * 8;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  auto fetch = [&](int row) {
    u32x4 v = *reinterpret_cast<const u32x4*>(wl + row * 256 + ((c ^ (row & 15)) << 4));
    if (row & 16) { unsigned t0 = v[0], t1 = v[1]; v[0] = v[2]; v[1] = v[3]; v[2] = t0; v[3] = t1; }
    return v;
  };
  if (mw + 128 <= M && nw + 128 <= N && (ldc & 7) == 0) {        // interior wave tile: 16-byte stores, no checks
    bf16_t* dst = C + (size_t)(mw + rsub) * ldc + n;
    const size_t step = (size_t)4 * ldc;
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
      *reinterpret_cast<u32x4*>(dst) = fetch(it * 4 + rsub);
      dst += step;
    }
  } else {
    for (int it = 0; it < 32; ++it) {
      const int row = it * 4 + rsub;
      const u32x4 v = fetch(row);
      const int m = mw + row;
      if (m < M) {
        bf16_t* dst = C + (size_t)m * ldc + n;
        if (n + 4 <= N) { u32x2 lo; lo[0] = v[0]; lo[1] = v[1]; *reinterpret_cast<u32x2*>(dst) = lo; }
        if (n + 8 <= N) { u32x2 hi; hi[0] = v[2]; hi[1] = v[3]; *reinterpret_cast<u32x2*>(dst + 4) = hi; }
      }
    }
  }
}

// Rotary embedding on the accumulators of a wave tile that is one attention head (128 columns starting at a multiple
// of 128): column c < 64 pairs with column c + 64, which the same lane holds in the same register of acc[i][j + 2]
// (j = 0, 1), so the rotation by position * theta_c happens in registers, in fp32, before the one conversion to bf16.
// table[pos * 64 + c] = (cos, sin); pos = row % seq.  Every lane reads the 32-byte pieces of its own row's table row
// straight from memory (the table stays in L2); staging the rows through LDS with coalesced loads measured slower.
__device__ __forceinline__ void rope_rotate_acc(f32x16_t (&acc)[4][4], const float2* __restrict__ table, int seq, int M,
                                                int mw, int lane) {
  const int khalf = lane >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = mw + i * 32 + (lane & 31);
    m = m < M ? m : M - 1;                                 // rows past the end are never stored; keep the table read in bounds
    const float4* row = reinterpret_cast<const float4*>(table + (size_t)(m % seq) * 64);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = j * 32 + g * 8 + khalf * 4;          // this lane's 4 consecutive frequencies
        const float4 t0 = row[c / 2], t1 = row[c / 2 + 1]; // (cos, sin) of c, c + 1 and of c + 2, c + 3
        const float cs[4] = {t0.x, t0.z, t1.x, t1.z}, sn[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = acc[i][j][g * 4 + e], hi = acc[i][j + 2][g * 4 + e];
          acc[i][j][g * 4 + e] = lo * cs[e] - hi * sn[e];
          acc[i][j + 2][g * 4 + e] = hi * cs[e] + lo * sn[e];
        }
      }
  }
}

// Epilogue of the gate / up projection with the MLP activation fused in.  B is in paired slabs, so the wave tile's
// columns 0..63 are gate columns base..base + 63 (base = 128 tile_n + 64 wn) and its columns 64..127 the up columns of
// the same indices: a = silu(gate) * up is formed from the fp32 accumulators.  Stored: gate and up (bf16) where the
// plain [gate | up] layout has them (GU[m][base + c], GU[m][f + base + c]) and a (bf16) at A[m][base + c]; each of
// the three is a 128-byte row segment.  32 rows at a time go through the wave's own LDS ([32][400 B]).
__device__ __forceinline__ void epilogue_swiglu_rows(f32x16_t (&acc)[4][4], char* smem, int wave, int lane, bf16_t* GU,
                                                     bf16_t* Aout, int M, int f, int ldgu, int mw, int base) {
  char* const wl = smem + wave * 32768;
  constexpr int RS = 400;                                  // row stride: 3 x 128 B + 16 (keeps 16-byte alignment)
  const int khalf = lane >> 5, r = lane & 31;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4_t og, ou, oa;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float gv = acc[i][j][g * 4 + e], uv = acc[i][j + 2][g * 4 + e];
          og[e] = (bf16_t)gv;
          ou[e] = (bf16_t)uv;
          // silu(g) u = g u / (1 + 2^(-g log2 e)): hardware exp2 and reciprocal (1 ulp each), far below bf16's 2^-9
          oa[e] = (bf16_t)(gv * uv * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896f * gv)));
        }
        const int cb = (j * 32 + g * 8 + khalf * 4) * 2;   // byte offset of the 4 columns within a 128-byte segment
        *reinterpret_cast<bf16x4_t*>(wl + r * RS + cb) = og;
        *reinterpret_cast<bf16x4_t*>(wl + r * RS + 128 + cb) = ou;
        *reinterpret_cast<bf16x4_t*>(wl + r * RS + 256 + cb) = oa;
      }
    // the wave reads back only what it wrote itself: no workgroup barrier (the compiler orders LDS accesses of a wave)
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int it = 0; it < 12; ++it) {                      // 32 rows x 24 chunks of 16 bytes
      const int q = it * 64 + lane, row = q / 24, cc = q % 24, seg = cc >> 3, w8 = (cc & 7) * 8;
      const u32x4 v = *reinterpret_cast<const u32x4*>(wl + row * RS + seg * 128 + (cc & 7) * 16);
      const int m = mw + i * 32 + row;
      if (m < M) {
        bf16_t* dst = seg == 2 ? Aout + (size_t)m * f + base + w8 : GU + (size_t)m * ldgu + (seg == 1 ? f : 0) + base + w8;
        *reinterpret_cast<u32x4*>(dst) = v;
      }
    }
  }
}

// f(std::integral_constant<int, P0>{}), ..., f(std::integral_constant<int, P1 - 1>{}): a loop whose index is a
// constant expression inside the body
template <int P0, class F, int... I>
__device__ __forceinline__ void for_range_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, P0 + I>{}), ...);
}
template <int P0, int P1, class F>
__device__ __forceinline__ void for_range(F&& f) {
  for_range_impl<P0>(f, std::make_integer_sequence<int, P1 - P0>{});
}

// Issue position (0..63 within a trip of the main loop) of the trip's n-th tile load: one ahead of every fourth
// MFMA; -1 = none at p
__device__ constexpr int load_at(int p) { return (p & 3) == 1 ? p >> 2 : -1; }

// One output tile.  TNL = false: A(m, k) at A[m * lda + k], B(n, k) at B[n * ldb + k].  TNL = true: A[k * lda + m],
// B[k * ldb + n].  pid = position of the tile in the problem's tile sequence (groups of 8 tile rows, walked
// column by column).
template <bool TNL, int EPI>
__device__ __forceinline__ void direct_tile(char* smem, const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                            void* __restrict__ Cv, const bf16_t* __restrict__ R, int M, int N, int K, int lda,
                                            int ldb, int ldc, int tiles_m, int tiles_n, unsigned a_bytes, unsigned b_bytes,
                                            int tile_m, int tile_n, bool b_slab = false, const GemmExtra& ex = GemmExtra()) {
  constexpr int BM = 256, BN = 256, WM = 2, WN = 2, TM = 4, TN = 4;
  constexpr int OPB = 32768;                    // one operand of one stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment q: 0..3 = A rows (i = q), 4..7 = B rows (j = q - 4).  Byte address of this lane's read within
  // a slot: NT one per k-step, TN one (k-step and k-quad are immediates: 8192 and 2048 bytes)
  constexpr int KS = TNL ? 1 : 4;
  int faddr[8][KS];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int first = q < 4 ? wm * (BM / WM) + q * 32 : wn * (BN / WN) + (q - 4) * 32;
    if (TNL) {
      const int khalf = lane >> 5, cgrp = (lane >> 4) & 1, e = (lane >> 2) & 3, r = lane & 3;
      const int c16 = (first + cgrp * 16 + r * 4) >> 3;
      faddr[q][0] = (khalf * 8 + e) * 512 + ((c16 ^ (e << 2)) << 4) + (r & 1) * 8;
    } else {
      const int row = first + (lane & 31), khalf = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) faddr[q][ks] = row * ROW_BYTES + (((ks * 2 + khalf) ^ swz(row)) << 4);
    }
  }
  // tile loads: 16 per wave and tile, t even -> A, t odd -> B, each 1 KB of LDS; voff = this lane's byte offset
  // within the k-tile (out of range for rows or columns past the operand), the k-tile offset is scalar
  unsigned voff[16];
  unsigned a_tile, b_tile;
  if (TNL) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = 2 * (wave * 8 + j) + (lane >> 5);
      const int c16 = (lane & 31) ^ ((k & 3) << 2);
      const int ca = m0 + c16 * 8, cb = n0 + c16 * 8;
      voff[2 * j] = ca < M ? (unsigned)k * (unsigned)lda * 2u + (unsigned)ca * 2u : 0xFFFFFF00u;
      voff[2 * j + 1] = cb < N ? (unsigned)k * (unsigned)ldb * 2u + (unsigned)cb * 2u : 0xFFFFFF00u;
    }
    a_tile = 64u * (unsigned)lda * 2u;
    b_tile = 64u * (unsigned)ldb * 2u;
  } else {
    const int lrow = lane >> 3, c0 = (lane & 7) ^ lrow;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned coff = (unsigned)((c0 ^ j) << 4);
      voff[2 * j] = (unsigned)(m0 + wave * 64 + j * 8 + lrow) * (unsigned)lda * 2u + coff;
      // B in slabs: the 256 rows x 64 columns of tile column tile_n and k-tile kt lie together (32 KB, row-major
      // inside), so one load instruction covers 1 KB of consecutive memory instead of 128 bytes of 8 rows each
      voff[2 * j + 1] = b_slab ? (unsigned)tile_n * (unsigned)(K / BK) * 32768u + (unsigned)(wave * 64 + j * 8 + lrow) * 128u + coff
                               : (unsigned)(n0 + wave * 64 + j * 8 + lrow) * (unsigned)ldb * 2u + coff;
    }
    a_tile = BK * 2;
    b_tile = b_slab ? 32768u : BK * 2;
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
  const i32x4_t ra = make_desc(A, a_bytes), rb = make_desc(B, b_bytes);
  const unsigned lds0 = (unsigned)(size_t)(lds_void_t*)smem;
  // load idx (0..7) of this wave for one operand of k-tile `tile` into the ring slot whose address, plus this
  // wave's 8 KB share, is `base`
  auto issue_one = [&](i32x4_t desc, unsigned base, int tile, bool is_b, auto idx_c) __attribute__((always_inline)) {
    constexpr int idx = decltype(idx_c)::value;
    const unsigned soff = tile * (is_b ? b_tile : a_tile);
    const unsigned vo = voff[2 * idx + (is_b ? 1 : 0)];
    asm volatile("s_add_u32 m0, %0, %4\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(base), "v"(vo), "s"(desc), "s"(soff), "n"(idx * 1024) : "memory", "m0", "scc");
  };
  const unsigned lds_wave = lds0 + wave * 8192;
  // descriptor of an operand for k-tile `tile`: past the last tile it has length zero (the load then moves nothing
  // from memory and zero-fills its slot, so the count of loads in flight is the same on every trip)
  auto desc_for = [&](i32x4_t d, int tile) __attribute__((always_inline)) {
    d[2] = tile < K / BK ? d[2] : 0;
    return d;
  };
  // LDS is a ring of five 32 KB slots which the operands take in the order A0 B0 A1 B1 A2 ... (operand u in slot
  // u % 5).  While tile kt is computed its two slots are read, the two that tile kt - 1 has left are refilled with
  // B of tile kt + 1 and A of tile kt + 2, and A of tile kt + 1 sits in the fifth.  The sync at the top of tile kt
  // wants both operands of tile kt landed: every load but this wave's last 8 (A of tile kt + 1), which stay in
  // flight across the barrier, so the memory pipe never runs empty.  The slots of a tile change from trip to
  // trip: cur[][] = LDS addresses of the fragments of the tile being read, rebuilt for the next tile
  // under the MFMAs of the last k-step that reads nothing any more.
  constexpr unsigned RING = 5 * OPB;
  auto two_on = [](unsigned off) __attribute__((always_inline)) { off += 2 * OPB; return off >= RING ? off - RING : off; };
  int cur[8][KS];
  i16x4_t fr[2][8][2];
  // half 0 / 1: the two 8-byte halves of fragment q (TN: one transposing read each; NT: one 16-byte read at half 0)
  auto load_half = [&](int set, int ks, int q, int half) __attribute__((always_inline)) {
    if (TNL) {
      fr[set][q][half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t*)(unsigned)(cur[q][0] + ks * 8192 + half * 2048));
    } else if (half == 0) {
      typedef short i16x8_t __attribute__((ext_vector_type(8)));
      typedef __attribute__((address_space(3))) i16x8_t lds_i16x8_t;
      const i16x8_t v = *(const lds_i16x8_t*)(unsigned)cur[q][TNL ? 0 : ks];
      fr[set][q][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
      fr[set][q][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
    }
  };
  auto frag = [&](int set, int q) __attribute__((always_inline)) {
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(fr[set][q][0], fr[set][q][1], 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // fragments are read in the order a0 b0 a1 b1 ...; the MFMA order uses the ones read first first
  constexpr int MI[16] = {0, 1, 0, 1, 2, 2, 0, 1, 2, 3, 3, 3, 0, 1, 2, 3};
  constexpr int MJ[16] = {0, 0, 1, 1, 0, 1, 2, 2, 2, 0, 1, 2, 3, 3, 3, 3};
  constexpr int LQ[8] = {0, 4, 1, 5, 2, 6, 3, 7};
  auto mma_one = [&](int set, int t) __attribute__((always_inline)) {
    acc[MI[t]][MJ[t]] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(set, 4 + MJ[t]), frag(set, MI[t]), acc[MI[t]][MJ[t]], 0, 0, 0);
  };
  // One trip of the loop = 64 MFMAs = 64 issue positions p: 0..15 are k-step 3 of the previous tile (fragment set
  // 1, in registers), 16..63 k-steps 0..2 of tile kt.  An MFMA occupies the matrix pipe for 32 cycles, which is
  // all the room there is for whatever the wave issues ahead of the next one; a tile load takes most of that by
  // itself (three scalar instructions and a 64-lane address), so no position carries more than one expensive
  // thing:
  //  * fragment reads (k-step 0 of tile kt during positions 0..15, then step s + 1 during step s; the reads of
  //    step 3 are all out by position 55), NT at even positions, TN one at every position;
  //  * the 16 tile loads of the trip, n = 0..7 = B of tile kt + 1 into the slot at pa, 8..15 = A of tile kt + 2
  //    into the slot at pb, at positions 1, 5, ..., 61 (for TN the read of such a position moves to the one before);
  //  * the fragment addresses of the next tile, rebuilt at positions 56..63 when nothing reads the old ones.
  // Loads issued back to back (16 by each of four waves at the same point) fill the address queue of the texture
  // unit, which blocks the waves that issue them and the MFMAs behind, and cost a third more L2 misses.
  auto reads_at = [&](int p, bool next) __attribute__((always_inline)) {
    if (p < 16) {
      if (!next) return;
      if (TNL) load_half(0, 0, LQ[p >> 1], p & 1);
      else if ((p & 1) == 0) load_half(0, 0, LQ[p >> 1], 0);
      return;
    }
    const int ks = (p - 16) >> 4, t = (p - 16) & 15, q = t >> 1, set = ks & 1;
    if (ks < 2) {
      if (TNL) load_half(set ^ 1, ks + 1, LQ[q], t & 1);
      else if ((t & 1) == 0) load_half(set ^ 1, ks + 1, LQ[q], 0);
    } else if (q < 4) {                            // last reads of these slots: all requested in the first half
      if (TNL) {
        load_half(set ^ 1, ks + 1, LQ[t], 0);
        load_half(set ^ 1, ks + 1, LQ[t], 1);
      } else if ((t & 1) == 0) {
        load_half(set ^ 1, ks + 1, LQ[t], 0);
        load_half(set ^ 1, ks + 1, LQ[t + 1], 0);
      }
    }
  };
  auto position = [&](auto p_c, unsigned na, unsigned nb, i32x4_t db, i32x4_t da, unsigned base_b, unsigned base_a, int kt,
                      bool refill, bool next) __attribute__((always_inline)) {
    constexpr int p = decltype(p_c)::value;
    constexpr int n = load_at(p), n1 = p < 63 ? load_at(p + 1) : -1;
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (n >= 0) {
      if (refill) {
        if constexpr (n < 8) issue_one(db, base_b, kt + 1, true, std::integral_constant<int, n>{});
        else issue_one(da, base_a, kt + 2, false, std::integral_constant<int, n - 8>{});
      }
    }
    if (!(TNL && n >= 0)) reads_at(p, next);
    if (TNL && n1 >= 0) reads_at(p + 1, next);
    if (p >= 56) {
      constexpr int PER = 8 * KS / 8;              // addresses per position
#pragma unroll
      for (int e = (p - 56) * PER; e < (p - 55) * PER; ++e) cur[e / KS][e % KS] = faddr[e / KS][e % KS] + (int)(lds0 + (e / KS < 4 ? na : nb));
    }
    __builtin_amdgcn_sched_barrier(0);
    if (p < 16) mma_one(1, p); else mma_one(((p - 16) >> 4) & 1, (p - 16) & 15);
  };
  // positions [p0, p1) of the trip of tile kt; pa, pb = byte offsets of the slots the previous tile has left
  auto trip = [&](auto p0, auto p1, unsigned pa, unsigned pb, unsigned na, unsigned nb, int kt, bool refill, bool next)
      __attribute__((always_inline)) {
    const i32x4_t db = desc_for(rb, kt + 1), da = desc_for(ra, kt + 2);
    const unsigned base_b = lds_wave + pa, base_a = lds_wave + pb;
    for_range<decltype(p0)::value, decltype(p1)::value>(
        [&](auto p) __attribute__((always_inline)) { position(p, na, nb, db, da, base_b, base_a, kt, refill, next); });
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr std::integral_constant<int, 0> P0{};
  constexpr std::integral_constant<int, 16> P16{};
  constexpr std::integral_constant<int, 64> P64{};
#define OPTSTAGE_TILE_SYNC(n) asm volatile("s_waitcnt vmcnt(" #n ") lgkmcnt(0)\n\ts_barrier" ::: "memory")
  const int nk = K / BK;
#pragma unroll
  for (int u = 0; u < 5; ++u) {
    const i32x4_t d = desc_for((u & 1) ? rb : ra, u >> 1);
    for_range<0, 8>([&](auto idx) __attribute__((always_inline)) { issue_one(d, lds_wave + u * OPB, u >> 1, (u & 1) != 0, idx); });
  }
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) cur[q][ks] = faddr[q][ks] + (int)(lds0 + (q < 4 ? 0 : OPB));
  OPTSTAGE_TILE_SYNC(24);
#pragma unroll
  for (int q = 0; q < 8; ++q) { load_half(0, 0, LQ[q], 0); load_half(0, 0, LQ[q], 1); }
  unsigned pa = 0, pb = OPB;                         // slots of the tile before tile kt
  trip(P16, P64, 0, 0, two_on(pa), two_on(pb), 0, false, true);
  for (int kt = 1; kt < nk; ++kt) {
    const unsigned oa = two_on(pa), ob = two_on(pb);
    OPTSTAGE_TILE_SYNC(8);
    trip(P0, P64, pa, pb, two_on(oa), two_on(ob), kt, true, true);
    pa = oa;
    pb = ob;
  }
  trip(P0, P16, 0, 0, 0, 0, 0, false, false);
  OPTSTAGE_TILE_SYNC(0);                             // every wave is done with the operand tiles, nothing in flight
#undef OPTSTAGE_TILE_SYNC
  if (EPI == EPI_ACCUM || EPI == EPI_STOREF) {
    epilogue_via_lds<EPI, TM, TN, 4>(acc, smem, wave, lane, Cv, R, M, N, ldc, m0 + wm * (BM / WM), n0 + wn * (BN / WN));
  } else if (EPI == EPI_SWIGLU) {
    epilogue_swiglu_rows(acc, smem, wave, lane, reinterpret_cast<bf16_t*>(Cv), reinterpret_cast<bf16_t*>(ex.a_out), M, ex.f, ldc,
                         m0 + wm * (BM / WM), tile_n * 128 + wn * 64);
  } else {
    if (EPI == EPI_ROPE && n0 + wn * (BN / WN) < ex.rot_cols)      // this wave's 128 columns are a q or k head
      rope_rotate_acc(acc, ex.table, ex.seq, M, m0 + wm * (BM / WM), lane);
    epilogue_bf16_rows<(EPI == EPI_ROPE ? EPI_STORE : EPI)>(acc, smem, wave, lane, reinterpret_cast<bf16_t*>(Cv), R, M, N, ldc,
                                                             m0 + wm * (BM / WM), n0 + wn * (BN / WN));
  }
}

// Consecutive hardware workgroup ids go to different XCDs: give every XCD one contiguous range of the sequence
__device__ __forceinline__ int xcd_remap(int id, int n) { return (n & 7) == 0 ? (id & 7) * (n >> 3) + (id >> 3) : id; }

// Which output tile workgroup `id` of a problem computes (id counted from the problem's first workgroup; n = the
// problem's tile count).
//  order 0: the tile sequence walks groups of 8 tile rows column by column, and every XCD takes one contiguous
//           eighth of it: the 32 tiles an XCD has in flight form an 8 x 4 patch that shares 12 operand panels in its
//           L2, but the eight XCDs work far apart and share nothing.
//  order 1: every round of 256 workgroups covers one 16 x 16 patch of tiles; XCD x (= id % 8) takes the 4 x 8 part
//           at rows 4 (x % 4), columns 8 (x / 4) of it (12 panels in its L2 as before), so the chip as a whole touches
//           32 panels per round instead of 96 and two thirds of the L2 misses can hit in the memory-side cache.
//           Tiles outside the whole patches (a strip on the right, one at the bottom) come last, column by column.
__device__ __forceinline__ void tile_coords(int id, int n, int tiles_m, int tiles_n, int order, int& tile_m, int& tile_n) {
  if (order == 1) {
    const int nfm = tiles_m >> 4, nfn = tiles_n >> 4, whole = nfm * nfn * 256;
    if (id < whole) {
      const int sp = id >> 8, x = id & 7, w = (id >> 3) & 31;
      tile_m = (sp % nfm) * 16 + (x & 3) * 4 + (w & 3);
      tile_n = (sp / nfm) * 16 + (x >> 2) * 8 + (w >> 2);
      return;
    }
    int q = id - whole;
    const int rn = tiles_n - nfn * 16, rm = tiles_m - nfm * 16;
    if (q < tiles_m * rn) { tile_m = q % tiles_m; tile_n = nfn * 16 + q / tiles_m; return; }
    q -= tiles_m * rn;
    tile_m = nfm * 16 + q % rm;
    tile_n = q / rm;
    return;
  }
  const int pid = xcd_remap(id, n);
  constexpr int GM = 8;
  const int grp = pid / (GM * tiles_n);
  const int first_m = grp * GM;
  const int gsz = min(tiles_m - first_m, GM);
  const int in_grp = pid - grp * GM * tiles_n;
  tile_m = first_m + in_grp % gsz;
  tile_n = in_grp / gsz;
}

template <bool TNL, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_direct_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                               void* __restrict__ Cv, const bf16_t* __restrict__ R, int M, int N,
                                                               int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n,
                                                               unsigned a_bytes, unsigned b_bytes, int b_slab, const GemmExtra ex,
                                                               int order) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int tile_m, tile_n;
  tile_coords(blockIdx.x, tiles_m * tiles_n, tiles_m, tiles_n, order, tile_m, tile_n);
  direct_tile<TNL, EPI>(smem, A, B, Cv, R, M, N, K, lda, ldb, ldc, tiles_m, tiles_n, a_bytes, b_bytes, tile_m, tile_n,
                        !TNL && b_slab != 0, ex);
}

// Several independent products with the same K in one launch (the weight-gradient GEMMs of a W op: four per
// layer, none depending on another): their tiles form one sequence, so the partly filled last round of
// workgroups that every product would leave behind on its own happens once.
constexpr int MAX_GROUP = 16;
struct GroupedProblem {
  const bf16_t* A; const bf16_t* B; void* C; const bf16_t* R;
  int M, N, lda, ldb, ldc, tiles_m, tiles_n, first_tile;
  unsigned a_bytes, b_bytes;
};
struct GroupedArgs { int n, K, total, order; GroupedProblem p[MAX_GROUP]; };

template <bool TNL, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_direct_grouped_kernel(const GroupedArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // order 1 within each problem: workgroups with equal (id - first_tile) % 8 are on one XCD whatever first_tile is,
  // and any 256 consecutive ids are in flight together, which is all the patch mapping relies on
  const int id = g.order == 1 ? (int)blockIdx.x : xcd_remap(blockIdx.x, g.total);
  int q = 0;
  for (int i = 1; i < g.n; ++i)
    if (id >= g.p[i].first_tile) q = i;
  const GroupedProblem& pr = g.p[q];
  int tile_m, tile_n;
  if (g.order == 1) {
    tile_coords(id - pr.first_tile, pr.tiles_m * pr.tiles_n, pr.tiles_m, pr.tiles_n, 1, tile_m, tile_n);
  } else {                                   // the sequence position is already XCD-mapped over the whole launch
    constexpr int GM = 8;
    const int pid = id - pr.first_tile, grp = pid / (GM * pr.tiles_n), first_m = grp * GM;
    const int gsz = min(pr.tiles_m - first_m, GM), in_grp = pid - grp * GM * pr.tiles_n;
    tile_m = first_m + in_grp % gsz;
    tile_n = in_grp / gsz;
  }
  direct_tile<TNL, EPI>(smem, pr.A, pr.B, pr.C, pr.R, pr.M, pr.N, g.K, pr.lda, pr.ldb, pr.ldc, pr.tiles_m, pr.tiles_n,
                        pr.a_bytes, pr.b_bytes, tile_m, tile_n);
}

// Measured on the weight-gradient set of the grouped-query stage (8 products, one launch): order 1 1229 TFLOP/s against
// 1187 for order 0 (TN with the fp32 read-add-store, whose operand panels are re-read most: 2.6 x the algorithmic bytes
// miss the L2); the NT products are within 0.5 % either way and keep order 0.
constexpr int tile_order(bool tnl) { return tnl ? 1 : 0; }

template <bool TNL, int EPI>
hipError_t launch_direct(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                         int ldc, hipStream_t s, bool b_slab = false, const GemmExtra& ex = GemmExtra()) {
  auto kern = gemm_bf16_direct_kernel<TNL, EPI>;
  constexpr int smem = 163840;
  static LdsAttrOnce lds_attr;
  if (hipError_t e = lds_attr.ensure(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
  // byte extent of each operand: whatever lies past it reads as zero
  const unsigned a_bytes = (unsigned)(TNL ? ((size_t)(K - 1) * lda + M) * 2 : ((size_t)(M - 1) * lda + K) * 2);
  const unsigned b_bytes = b_slab ? (unsigned)((size_t)tiles_n * (K / 64) * 32768)
                                  : (unsigned)(TNL ? ((size_t)(K - 1) * ldb + N) * 2 : ((size_t)(N - 1) * ldb + K) * 2);
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, s, (const bf16_t*)A, (const bf16_t*)B, C, (const bf16_t*)R,
                     M, N, K, lda, ldb, ldc, tiles_m, tiles_n, a_bytes, b_bytes, b_slab ? 1 : 0, ex, tile_order(TNL));
  return hipGetLastError();
}

// the direct path needs whole 64-wide k-tiles and 32-bit byte offsets (NT: including the rows a partial edge
// tile reaches past the operand)
bool direct_applies(bool tnl, int M, int N, int K, int lda, int ldb) {
  if (K % 64) return false;
  const unsigned long long lim = 0xF0000000ull;
  if (tnl) return ((unsigned long long)K * lda * 2 < lim) && ((unsigned long long)K * ldb * 2 < lim);
  return ((unsigned long long)(M + 256) * lda * 2 < lim) && ((unsigned long long)(N + 256) * ldb * 2 < lim);
}
template <bool TNL, int EPI>
hipError_t launch_direct_grouped(int n, const GemmProblem* pr, int K, hipStream_t s) {
  auto kern = gemm_bf16_direct_grouped_kernel<TNL, EPI>;
  constexpr int smem = 163840;
  static LdsAttrOnce lds_attr;
  if (hipError_t e = lds_attr.ensure(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  GroupedArgs g;
  g.n = n;
  g.K = K;
  int total = 0;
  for (int i = 0; i < n; ++i) {
    GroupedProblem& q = g.p[i];
    q.A = (const bf16_t*)pr[i].A; q.B = (const bf16_t*)pr[i].B; q.C = pr[i].C; q.R = (const bf16_t*)pr[i].R;
    q.M = pr[i].M; q.N = pr[i].N; q.lda = pr[i].lda; q.ldb = pr[i].ldb; q.ldc = pr[i].ldc;
    q.tiles_m = (q.M + 255) / 256;
    q.tiles_n = (q.N + 255) / 256;
    q.first_tile = total;
    total += q.tiles_m * q.tiles_n;
    q.a_bytes = (unsigned)(TNL ? ((size_t)(K - 1) * q.lda + q.M) * 2 : ((size_t)(q.M - 1) * q.lda + K) * 2);
    q.b_bytes = (unsigned)(TNL ? ((size_t)(K - 1) * q.ldb + q.N) * 2 : ((size_t)(q.N - 1) * q.ldb + K) * 2);
  }
  g.total = total;
  g.order = tile_order(TNL);
  hipLaunchKernelGGL(kern, dim3(total), dim3(256), smem, s, g);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, bool A_RC, bool B_RC, int EPI>
hipError_t launch_cfg(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                      int ldc, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, A_RC, B_RC, EPI>;
  constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
  static LdsAttrOnce lds_attr;
  if (hipError_t e = lds_attr.ensure(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WM * WN), smem, s, (const bf16_t*)A, (const bf16_t*)B, C,
                     (const bf16_t*)R, M, N, K, lda, ldb, ldc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool RC, int EPI>
hipError_t launch_layout(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                         int ldc, hipStream_t s) {
  long big_tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 128) {
    if (direct_applies(RC, M, N, K, lda, ldb)) return launch_direct<RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    // register-staged path: 8 waves (4 x 2) for the transposing TN loader, 4 waves (2 x 2) otherwise
    if constexpr (RC) {
      return launch_cfg<256, 256, 4, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    } else {
      return launch_cfg<256, 256, 2, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    }
  }
  return launch_cfg<128, 128, 2, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
}

}  // namespace

// B in slabs is served by the direct kernel only: shapes that the dispatcher would send elsewhere do not qualify
bool gemm_bf16_slab_applies(int M, int N, int K, int lda) {
  if (M <= 0 || N <= 0 || K <= 0 || (K % 64) || (lda & 7) || (N & 3)) return false;
  const long tiles_n = (N + 255) / 256, big_tiles = (long)((M + 255) / 256) * tiles_n;
  if (big_tiles < 128 || (unsigned long long)tiles_n * (K / 64) * 32768ull >= 0xF0000000ull) return false;
  return direct_applies(false, M, N, K, lda, 8);
}

// The fused epilogues run on the direct kernel only, on whole heads / whole gate-up pairs: what must hold for them
bool gemm_bf16_fused_applies(int epi, int M, int N, int K, int lda, int head_dim) {
  if (epi == EPI_ROPE) return head_dim == 128 && (N % 128) == 0 && (N & 3) == 0 && direct_applies(false, M, N, K, lda, K) &&
                              (long)((M + 255) / 256) * ((N + 255) / 256) >= 128 && (lda & 7) == 0 && (K % 64) == 0;
  if (epi == EPI_SWIGLU) return (N % 256) == 0 && gemm_bf16_slab_applies(M, N, K, lda);
  return false;
}

hipError_t launch_gemm_bf16(int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                            int K, int lda, int ldb, int ldc, hipStream_t s, const GemmExtra* extra) {
  // host-side shape checks: 16-byte vector accesses need these
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  if (epi == EPI_ROPE) {
    // whole heads per wave tile, rotated columns a whole number of heads, table and sequence length given
    if (!extra || !extra->table || extra->seq <= 0 || extra->rot_cols < 0 || extra->rot_cols > N || (extra->rot_cols % 128) ||
        (ldc & 7) || (layout != GEMM_NT && layout != GEMM_NT_SLAB) || !gemm_bf16_fused_applies(epi, M, N, K, lda, 128))
      return hipErrorInvalidValue;
    if (layout == GEMM_NT_SLAB) {
      if (!gemm_bf16_slab_applies(M, N, K, lda)) return hipErrorInvalidValue;
      return launch_direct<false, EPI_ROPE>(A, B, C, R, M, N, K, lda, 64, ldc, s, true, *extra);
    }
    if ((ldb & 7) || ldb < K) return hipErrorInvalidValue;
    return launch_direct<false, EPI_ROPE>(A, B, C, R, M, N, K, lda, ldb, ldc, s, false, *extra);
  }
  if (epi == EPI_SWIGLU) {
    // N = 2 f columns in paired slabs; GU rows of ldc elements, a rows of f elements, 16-byte row segments
    if (!extra || !extra->a_out || extra->f <= 0 || N != 2 * extra->f || (extra->f % 128) || (ldc & 7) || ldc < N ||
        layout != GEMM_NT_SLAB || !gemm_bf16_fused_applies(epi, M, N, K, lda, 0))
      return hipErrorInvalidValue;
    return launch_direct<false, EPI_SWIGLU>(A, B, C, R, M, N, K, lda, 64, ldc, s, true, *extra);
  }
  if (layout == GEMM_NT_SLAB) {
    if ((ldc & 3) || !gemm_bf16_slab_applies(M, N, K, lda)) return hipErrorInvalidValue;
    if (epi == EPI_STORE) return launch_direct<false, EPI_STORE>(A, B, C, R, M, N, K, lda, 64, ldc, s, true);
    if (epi == EPI_RESID) return launch_direct<false, EPI_RESID>(A, B, C, R, M, N, K, lda, 64, ldc, s, true);
    return hipErrorInvalidValue;
  }
  if ((lda & 7) || (ldb & 7) || (ldc & 3) || (N & 3)) return hipErrorInvalidValue;
  if (layout == GEMM_NT) {
    if (K & 7) return hipErrorInvalidValue;
    if (epi == EPI_STORE) return launch_layout<false, EPI_STORE>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    if (epi == EPI_RESID) return launch_layout<false, EPI_RESID>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    if (epi == EPI_ACCUM) return launch_layout<false, EPI_ACCUM>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
  } else if (layout == GEMM_TN) {
    if ((M & 7) || (N & 7)) return hipErrorInvalidValue;
    if (epi == EPI_STORE) return launch_layout<true, EPI_STORE>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    if (epi == EPI_ACCUM) return launch_layout<true, EPI_ACCUM>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    if (epi == EPI_STOREF) return launch_layout<true, EPI_STOREF>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
  }
  return hipErrorInvalidValue;
}

// n independent products sharing layout, epilogue and K in one launch: whether the set qualifies (every product
// on the direct path, operands aligned as the kernels need, at least half a round of tiles in total)
bool gemm_bf16_grouped_applies(int layout, int n, const GemmProblem* pr, int K) {
  if (n <= 0 || n > MAX_GROUP || K <= 0 || (K % 64)) return false;
  long tiles = 0;
  for (int i = 0; i < n; ++i) {
    const GemmProblem& q = pr[i];
    if (q.M <= 0 || q.N <= 0) return false;
    if ((q.lda & 7) || (q.ldb & 7) || (q.ldc & 3) || (q.N & 3)) return false;
    if (layout == GEMM_TN && ((q.M & 7) || (q.N & 7))) return false;
    if (!direct_applies(layout == GEMM_TN, q.M, q.N, K, q.lda, q.ldb)) return false;
    tiles += (long)((q.M + 255) / 256) * ((q.N + 255) / 256);
  }
  return tiles >= 128;
}

hipError_t launch_gemm_bf16_grouped(int layout, int epi, int n, const GemmProblem* pr, int K, hipStream_t s) {
  if (!gemm_bf16_grouped_applies(layout, n, pr, K)) return hipErrorInvalidValue;
  if (layout == GEMM_TN && epi == EPI_ACCUM) return launch_direct_grouped<true, EPI_ACCUM>(n, pr, K, s);
  if (layout == GEMM_TN && epi == EPI_STORE) return launch_direct_grouped<true, EPI_STORE>(n, pr, K, s);
  if (layout == GEMM_TN && epi == EPI_STOREF) return launch_direct_grouped<true, EPI_STOREF>(n, pr, K, s);
  if (layout == GEMM_NT && epi == EPI_STORE) return launch_direct_grouped<false, EPI_STORE>(n, pr, K, s);
  if (layout == GEMM_NT && epi == EPI_ACCUM) return launch_direct_grouped<false, EPI_ACCUM>(n, pr, K, s);
  return hipErrorInvalidValue;
}
