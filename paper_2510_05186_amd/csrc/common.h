// Shared device/host helpers for the optstage kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

// Raises a kernel's dynamic LDS limit, once per device (the attribute belongs to the function on one device; a
// process that drives several GPUs needs it on each).  One slot of flags per kernel at the call site.
struct LdsAttrOnce {
  std::atomic<unsigned long long> done{0};        // bit d: set on device d (devices past 63 set it on every launch)
  hipError_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = dev < 64 ? 1ull << dev : 0ull;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
  }
};

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

enum { DT_FP32 = 0, DT_BF16 = 1 };
enum { FAM_GPT = 0, FAM_LLAMA = 1 };

// GEMM operand layouts: C[M,N] = sum_k A(m,k) * B(n,k)
//   NT: A is [M,K] row-major, B is [N,K] row-major  (both contiguous along the contraction)
//   TN: A is [K,M] row-major, B is [K,N] row-major  (both contiguous along their output index)
// GEMM_NT_SLAB: C = A B^T with B stored in slabs of 256 rows x 64 columns, slab (n / 256, k / 64) at element offset
// ((n / 256) * (K / 64) + k / 64) * 16384, row-major inside, rows padded to a multiple of 256
enum { GEMM_NT = 0, GEMM_TN = 1, GEMM_NT_SLAB = 2 };
// epilogues: store C (stage dtype); store C + R (R like C); C (fp32) += product; C (fp32) = product;
// EPI_ROPE: store C with the q and k head columns rotated by position (rotary embedding fused into the QKV projection);
// EPI_SWIGLU: B holds the gate / up weight in paired slabs (GEMM_NT_SLAB with rows paired, see launch_slabs): stores the
// product in the plain [gate | up] layout AND a = silu(gate) * up (the MLP activation fused into the gate / up projection)
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_ACCUM = 2, EPI_STOREF = 3, EPI_ROPE = 4, EPI_SWIGLU = 5 };
// what the two fused epilogues need beyond C: the rotary table [seq][64] (cos, sin), the sequence length (position =
// row % seq) and the number of leading columns that are q / k heads; the activation output [M, f] and f
struct GemmExtra {
  const float2* table = nullptr; int seq = 0; int rot_cols = 0;
  void* a_out = nullptr; int f = 0;
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// 16-byte vector of T (4 floats or 8 bf16) with element access in fp32
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  f32x4_t v;
  __device__ __forceinline__ float get(int i) const { return v[i]; }
  __device__ __forceinline__ void set(int i, float x) { v[i] = x; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  bf16x8_t v;
  __device__ __forceinline__ float get(int i) const { return (float)v[i]; }
  __device__ __forceinline__ void set(int i, float x) { v[i] = (bf16_t)x; }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// launchers implemented in the .hip files; all return hipError_t from the launch
int attn_dkv_split(int seq, int batch, int n_q, int n_kv);
struct GemmProblem { const void* A; const void* B; void* C; const void* R; int M, N, lda, ldb, ldc; };
bool gemm_bf16_grouped_applies(int layout, int n, const GemmProblem* problems, int K);
hipError_t launch_gemm_bf16_grouped(int layout, int epi, int n, const GemmProblem* problems, int K, hipStream_t s);
hipError_t launch_gemm_bf16(int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                            int K, int lda, int ldb, int ldc, hipStream_t s, const GemmExtra* extra = nullptr);
bool gemm_bf16_fused_applies(int epi, int M, int N, int K, int lda, int head_dim);
hipError_t launch_gemm_f32(int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                           int K, int lda, int ldb, int ldc, hipStream_t s);
hipError_t launch_norm_fwd(int dtype, int family, const void* x, const void* gamma, const void* beta, void* out,
                           float* stats, int rows, int h, float eps, hipStream_t s);
hipError_t launch_norm_bwd(int dtype, int family, const void* dn, const void* x, const float* stats,
                           const void* gamma, const void* dres, void* dx, float* partial, float* dgamma,
                           float* dbeta, int rows, int h, hipStream_t s, int overwrite = 0);
int norm_bwd_partial_rows(int rows);
hipError_t launch_act_fwd(int dtype, int family, const void* gu, void* a, int rows, int f, hipStream_t s);
hipError_t launch_act_bwd(int dtype, int family, const void* da, const void* gu, void* dgu, int rows, int f,
                          hipStream_t s);
hipError_t launch_rope_table(float* table, int seq, int d, float base, hipStream_t s);
hipError_t launch_rope(int dtype, const void* src, void* dst, const float* table, int rows, int seq, int n_q, int n_kv,
                       int d, int backward, int do_rotate, hipStream_t s);
hipError_t launch_transpose(int dtype, const void* src, void* dst, int rows, int cols, hipStream_t s);
// bf16 weight into the slab layout of GEMM_NT_SLAB: B[n][k] = src[n * K + k], or src[k * N + n] when transposed = 1.
// transposed = 2 (paired): src is a [gate | up] weight of N = 2 f rows; slab row 256 t + 128 w + 64 q + o holds source
// row q f + 128 t + 64 w + o, so that each wave of an output tile owns 64 gate columns and the 64 matching up columns
// (f % 128 == 0)
hipError_t launch_slabs(const void* src, void* dst, int N, int K, int transposed, hipStream_t s);
bool gemm_bf16_slab_applies(int M, int N, int K, int lda);
hipError_t launch_checksum(const void* buf, uint64_t bytes, uint64_t* out_dev, hipStream_t s);
hipError_t launch_attn_fwd(int dtype, const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv,
                           int d, hipStream_t s);
// ws: fp32 scratch of attn_bwd_ws_floats() elements
hipError_t launch_attn_bwd(int dtype, const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv,
                           float* ws, int seq, int batch, int n_q, int n_kv, int d, hipStream_t s);
uint64_t attn_bwd_ws_floats(int seq, int batch, int n_q, int n_kv, int d);
