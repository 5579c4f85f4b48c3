// bf16 MFMA GEMM for gfx950: C[M,N] = sum_k A(m,k) * B(n,k), fp32 accumulation.
//
// These are the three linear maps of a stage (paper Sec. 2.2): forward Y = X W^T (NT), backward for
// activations dX = dY W (NT against the transposed weight copy), backward for weights dW += dY^T X (TN).
//
// Design (CDNA4): one workgroup of 4 waves (2 x 2) owns a BM x BN output tile; the K loop advances
// 64 elements at a time through double-buffered LDS tiles (global -> registers -> LDS, one barrier per
// step).  LDS tiles are always [row][64 k] with the 16-byte chunk index XOR-swizzled by the row so that
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
template <int R_T> struct StageKC {
  static constexpr int NCH = R_T / 32;
  uint4 reg[NCH];
  __device__ __forceinline__ void load(const bf16_t* p, int ld, int row0, int rows, int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int q = tid + 256 * i;
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
      int q = tid + 256 * i;
      int row = q >> 3, c = q & 7;
      *reinterpret_cast<uint4*>(lds + row * ROW_BYTES + ((c ^ swz(row)) << 4)) = reg[i];
    }
  }
};

// Row-contiguous operand: element (r, k) at p[k * ld + r].  Thread gathers KV k-rows x 8 r and writes
// 8 pieces of KV k-contiguous elements.
template <int R_T> struct StageRC {
  static constexpr int KV = R_T / 32;   // 8 for 256-row tiles, 4 for 128-row tiles
  uint4 reg[KV];
  __device__ __forceinline__ static void coords(int tid, int& rc, int& kg) {
    if (R_T == 256) {
      rc = tid & 31;
      kg = tid >> 5;
    } else {
      rc = (tid & 7) | (((tid >> 4) & 1) << 3);
      kg = ((tid >> 3) & 1) | ((tid >> 5) << 1);
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

template <int R_T, bool RC> struct StageSel { typedef StageKC<R_T> type; };
template <int R_T> struct StageSel<R_T, true> { typedef StageRC<R_T> type; };

// ---- kernel ---------------------------------------------------------------------------------------
template <int BM, int BN, bool A_RC, bool B_RC, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                        void* __restrict__ Cv, const bf16_t* __restrict__ R, int M,
                                                        int N, int K, int lda, int ldb, int ldc, int tiles_m,
                                                        int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, BUF = A_BYTES + B_BYTES;
  constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 MFMA tiles per wave in m and n

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // XCD-aware tile order: consecutive hardware ids go to different XCDs, so give every XCD one
  // contiguous range of the tile sequence, and walk that sequence in groups of 4 tile rows.
  int pid = blockIdx.x;
  const int nblk = tiles_m * tiles_n;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  constexpr int GM = 4;
  const int grp = pid / (GM * tiles_n);
  const int first_m = grp * GM;
  const int gsz = min(tiles_m - first_m, GM);
  const int in_grp = pid - grp * GM * tiles_n;
  const int tile_m = first_m + in_grp % gsz, tile_n = in_grp / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  typename StageSel<BM, A_RC>::type sa;
  typename StageSel<BN, B_RC>::type sb;

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
    int row = wm * (BM / 2) + i * 32 + (lane & 31);
    a_off[i] = row * ROW_BYTES;
    a_sw[i] = swz(row);
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    int row = wn * (BN / 2) + j * 32 + (lane & 31);
    b_off[j] = A_BYTES + row * ROW_BYTES;
    b_sw[j] = swz(row);
  }
  const int khalf = lane >> 5;

  const int nk = (K + BK - 1) / BK;
  sa.load(A, lda, m0, M, 0, K, tid);
  sb.load(B, ldb, n0, N, 0, K, tid);
  sa.store(smem, tid);
  sb.store(smem + A_BYTES, tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt & 1) * BUF;
    char* nxt = smem + ((kt + 1) & 1) * BUF;
    const bool more = kt + 1 < nk;
    if (more) {
      sa.load(A, lda, m0, M, (kt + 1) * BK, K, tid);
      sb.load(B, ldb, n0, N, (kt + 1) * BK, K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8_t af[TM], bfr[TN];
      const int chunk = ks * 2 + khalf;
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(cur + a_off[i] + ((chunk ^ a_sw[i]) << 4));
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(cur + b_off[j] + ((chunk ^ b_sw[j]) << 4));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    if (more) {
      sa.store(nxt, tid);
      sb.store(nxt + A_BYTES, tid);
    }
    __syncthreads();
  }

  // epilogue: lane owns m = .. + (lane & 31) and, per register group g, n = .. + 8 g + 4 (lane >> 5) + 0..3
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * (BM / 2) + i * 32 + (lane & 31);
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * (BN / 2) + j * 32 + g * 8 + khalf * 4;
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

template <int BM, int BN, bool A_RC, bool B_RC, int EPI>
hipError_t launch_cfg(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                      int ldc, hipStream_t s) {
  auto kern = gemm_bf16_kernel<BM, BN, A_RC, B_RC, EPI>;
  constexpr int smem = 2 * (BM + BN) * ROW_BYTES;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), smem, s, (const bf16_t*)A, (const bf16_t*)B, C,
                     (const bf16_t*)R, M, N, K, lda, ldb, ldc, tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool RC, int EPI>
hipError_t launch_layout(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                         int ldc, hipStream_t s) {
  long big_tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 128)
    return launch_cfg<256, 256, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
  return launch_cfg<128, 128, RC, RC, EPI>(A, B, C, R, M, N, K, lda, ldb, ldc, s);
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
