// bf16 MFMA GEMM for gfx950: C[M,N] = sum_k A(m,k) * B(n,k), fp32 accumulation.
//
// These are the three linear maps of a stage (paper Sec. 2.2): forward Y = X W^T (NT), backward for
// activations dX = dY W (NT against the transposed weight copy), backward for weights dW += dY^T X (TN).
//
// Design (CDNA4): one workgroup of 4 or 8 waves owns a BM x BN output tile (256 x 256 for large problems);
// the K loop advances 64 elements at a time through double-buffered LDS tiles with one barrier per step.
// NT problems with K % 64 == 0 load their tiles straight from global memory into LDS (no registers, no
// ds_write); everything else stages tiles global -> registers -> LDS.  LDS tiles are always [row][64 k] with the 16-byte chunk index XOR-swizzled by the row so that
// both the 16-byte operand reads of v_mfma_f32_32x32x16_bf16 and the tile writes are bank-conflict
// free.  Operands that are contiguous along their output index (TN) are transposed in registers on the
// way into LDS (each thread gathers a KV x 8 patch and writes 8 k-contiguous pieces), so the MFMA read
// path is identical for every layout.  The MFMA is issued with the B fragment as its first operand:
// each lane then owns 4 consecutive n of one m, which gives 8-byte (bf16) / 16-byte (fp32) row-major
// global accesses in the epilogue.  Workgroup ids are remapped so that the tiles resident on one XCD
// (ids congruent mod 8) form a compact patch of the output and share A/B panels in that XCD's L2.
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
  char* const wl = smem + wave * SLICE;
  const int khalf = lane >> 5;
#pragma unroll
  for (int pass = 0; pass < TM / IPP; ++pass) {
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
    const int c = lane & 31;
    const int n = nw + c * 4;
#pragma unroll 4
    for (int p2 = 0; p2 < 16 * IPP; ++p2) {
      const int row = 2 * p2 + khalf;
      const int m = mw + pass * IPP * 32 + row;
      f32x4_t v = *reinterpret_cast<const f32x4_t*>(wl + row * 512 + ((c ^ (row & 31)) << 4));
      if (m < M && n < N) {
        const size_t off = (size_t)m * ldc + n;
        if (EPI == EPI_ACCUM) {
          float* C = reinterpret_cast<float*>(Cv);
          f32x4_t o = *reinterpret_cast<const f32x4_t*>(C + off);
          o[0] += v[0]; o[1] += v[1]; o[2] += v[2]; o[3] += v[3];
          *reinterpret_cast<f32x4_t*>(C + off) = o;
        } else {
          if (EPI == EPI_RESID) {
            bf16x4_t r = *reinterpret_cast<const bf16x4_t*>(R + off);
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
        if (EPI == EPI_ACCUM) {
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

// ---- NT kernel with direct global -> LDS tile loads -------------------------------------------------
// Same tile shape (256 x 256 x 64, 2 x 2 waves), LDS layout, fragment pipeline and epilogue as above, but
// the tiles never pass through registers: every wave issues 16 `buffer_load_dwordx4 ... lds` per k-tile,
// each filling 1 KB of LDS (lane i writes 16 bytes at base + 16 i).  The XOR swizzle is realised by the
// choice of the global address each lane loads (lane i of the load for tile rows 8 q .. 8 q + 7 fetches
// row 8 q + i / 8, logical chunk (i % 8) ^ swizzle(row)).  Rows past M or N read as zero through the
// buffer range check.  Requires K % 64 == 0 and operands below 4 GiB (checked on the host).
typedef __attribute__((address_space(3))) void lds_void_t;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_nt_lds_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                               void* __restrict__ Cv, const bf16_t* __restrict__ R, int M, int N,
                                                               int K, int lda, int ldb, int ldc, int tiles_m, int tiles_n,
                                                               unsigned a_bytes, unsigned b_bytes) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int BM = 256, BN = 256, WM = 2, WN = 2, TM = 4, TN = 4;
  constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, BUF = A_BYTES + B_BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

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

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

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
  // tile loads: wave w fills LDS rows 64 w .. 64 w + 63 of each operand, 8 rows per instruction
  __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(A), 0, a_bytes, 0x00020000);
  __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(B), 0, b_bytes, 0x00020000);
  const int lrow = lane >> 3, c0 = (lane & 7) ^ lrow;
  const unsigned a_row_off = (unsigned)(m0 + wave * 64 + lrow) * (unsigned)lda * 2u;
  const unsigned b_row_off = (unsigned)(n0 + wave * 64 + lrow) * (unsigned)ldb * 2u;
  const unsigned a_step = 8u * (unsigned)lda * 2u, b_step = 8u * (unsigned)ldb * 2u;
  auto issue_tile = [&](char* buf, int k0) {
    const int soff = k0 * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned coff = (unsigned)((c0 ^ j) << 4);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void_t*)(buf + (wave * 8 + j) * 1024), 16, a_row_off + j * a_step + coff, soff, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_t*)(buf + A_BYTES + (wave * 8 + j) * 1024), 16, b_row_off + j * b_step + coff, soff, 0, 0);
    }
  };
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

  const int nk = K / BK;
  char* const buf0 = smem;
  char* const buf1 = smem + BUF;
  issue_tile(buf0, 0);
  if (nk > 1) issue_tile(buf1, BK);
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  bf16x8_t fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  load_frags(fa0, fb0, buf0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = (kt & 1) ? buf1 : buf0;
    char* nxt = (kt & 1) ? buf0 : buf1;
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
    // tile kt+1 (issued one iteration ago) has landed in nxt and every read of cur has been issued
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (kt + 2 < nk) issue_tile(cur, (kt + 2) * BK);
    __builtin_amdgcn_sched_barrier(0);
    load_frags(fa0, fb0, nxt, 0);
    __builtin_amdgcn_sched_barrier(0);
    mma(fa1, fb1);
  }

  __syncthreads();                                   // every wave is done with the operand tiles
  epilogue_via_lds<EPI, TM, TN, 4>(acc, smem, wave, lane, Cv, R, M, N, ldc, m0 + wm * (BM / WM), n0 + wn * (BN / WN));
}

template <int EPI>
hipError_t launch_nt_lds(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                         int ldc, hipStream_t s) {
  auto kern = gemm_bf16_nt_lds_kernel<EPI>;
  constexpr int smem = 2 * 512 * ROW_BYTES;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256;
  // byte extent of each operand: rows past the end fall outside the buffer range and read as zero
  const unsigned a_bytes = (unsigned)(((size_t)(M - 1) * lda + K) * 2), b_bytes = (unsigned)(((size_t)(N - 1) * ldb + K) * 2);
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, s, (const bf16_t*)A, (const bf16_t*)B, C, (const bf16_t*)R,
                     M, N, K, lda, ldb, ldc, tiles_m, tiles_n, a_bytes, b_bytes);
  return hipGetLastError();
}

// the direct path needs whole 64-wide k-tiles and 32-bit byte offsets, including the rows a partial edge
// tile reaches past the operand
bool nt_lds_applies(int M, int N, int K, int lda, int ldb) {
  if (K % 64) return false;
  const unsigned long long lim = 0xF0000000ull;
  return ((unsigned long long)(M + 256) * lda * 2 < lim) && ((unsigned long long)(N + 256) * ldb * 2 < lim);
}
template <int BM, int BN, int WM, int WN, bool A_RC, bool B_RC, int EPI>
hipError_t launch_cfg(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                      int ldc, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, A_RC, B_RC, EPI>;
  constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
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
    // register-staged path: 8 waves (4 x 2) for the transposing TN loader, 4 waves (2 x 2) otherwise
    if constexpr (RC) {
      return launch_cfg<256, 256, 4, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    } else {
      if (nt_lds_applies(M, N, K, lda, ldb)) return launch_nt_lds<EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
      return launch_cfg<256, 256, 2, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
    }
  }
  return launch_cfg<128, 128, 2, 2, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
}

}  // namespace

hipError_t launch_gemm_bf16(int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                            int K, int lda, int ldb, int ldc, hipStream_t s) {
  // host-side shape checks: 16-byte vector accesses need these
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
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
  }
  return hipErrorInvalidValue;
}
