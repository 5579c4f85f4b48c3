// Single-kernel C-ABI entry points (include/optstage_ops.h) and the attention dispatch between the
// MFMA kernels and the general path.
#include <mutex>

#include "../../include/optstage_ops.h"
#include "common.h"

int optstage_fail_(int status, const char* msg);
hipError_t launch_attn_fwd_simple(int dtype, const void* qkv, void* o, float* lse, int seq, int batch, int n_q,
                                  int n_kv, int d, hipStream_t s);
hipError_t launch_attn_bwd_simple(int dtype, const void* qkv, const void* o, const void* dout, const float* lse,
                                  void* dqkv, float* ws, int seq, int batch, int n_q, int n_kv, int d, hipStream_t s);

bool attn_mfma_applies(int dtype, int d, int seq, int n_q, int n_kv);
hipError_t launch_attn_fwd_mfma(const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv, hipStream_t s);
hipError_t launch_attn_bwd_mfma(const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv, float* ws,
                                int seq, int batch, int n_q, int n_kv, hipStream_t s);

hipError_t launch_attn_fwd(int dtype, const void* qkv, void* o, float* lse, int seq, int batch, int n_q, int n_kv,
                           int d, hipStream_t s) {
  if (seq <= 0 || batch <= 0 || n_q <= 0 || n_kv <= 0 || n_q % n_kv) return hipErrorInvalidValue;
  if (attn_mfma_applies(dtype, d, seq, n_q, n_kv)) return launch_attn_fwd_mfma(qkv, o, lse, seq, batch, n_q, n_kv, s);
  return launch_attn_fwd_simple(dtype, qkv, o, lse, seq, batch, n_q, n_kv, d, s);
}

hipError_t launch_attn_bwd(int dtype, const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv,
                           float* ws, int seq, int batch, int n_q, int n_kv, int d, hipStream_t s) {
  if (seq <= 0 || batch <= 0 || n_q <= 0 || n_kv <= 0 || n_q % n_kv) return hipErrorInvalidValue;
  if (attn_mfma_applies(dtype, d, seq, n_q, n_kv)) return launch_attn_bwd_mfma(qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, s);
  return launch_attn_bwd_simple(dtype, qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, d, s);
}

uint64_t attn_bwd_ws_floats(int seq, int batch, int n_q, int n_kv, int d) {
  // D_t = <dO_t, O_t> per query row and head, then (grouped-query attention on the MFMA path only) the fp32
  // partials of dK, dV of the workgroups that share a kv head
  uint64_t n = (uint64_t)batch * n_q * seq;
  if (d == 128 && n_kv > 0 && n_q % n_kv == 0) {
    const int split = attn_dkv_split(seq, batch, n_q, n_kv);
    if (split > 1) n += (uint64_t)split * batch * seq * n_kv * 2 * d;
  }
  return n;
}

namespace {
optstage_status wrap(hipError_t e, const char* what) {
  if (e == hipSuccess) return OPTSTAGE_OK;
  char msg[256];
  snprintf(msg, sizeof msg, "%s: %s", what, hipGetErrorString(e));
  return (optstage_status)optstage_fail_(e == hipErrorInvalidValue ? OPTSTAGE_E_ARG : OPTSTAGE_E_HIP, msg);
}
bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
#define REQ(cond, what) \
  if (!(cond)) return (optstage_status)optstage_fail_(OPTSTAGE_E_ARG, what)
}  // namespace

extern "C" {

optstage_status optstage_op_gemm(uint32_t dtype, uint32_t layout, uint32_t epilogue, const void* A, const void* B,
                                 void* C, const void* R, uint32_t M, uint32_t N, uint32_t K, uint32_t lda,
                                 uint32_t ldb, uint32_t ldc, void* stream) {
  REQ(A && B && C && (epilogue != 1 || R), "gemm: null operand");
  REQ(aligned16(A) && aligned16(B) && aligned16(C) && aligned16(R), "gemm: operands must be 16-byte aligned");
  REQ(dtype <= 1 && layout <= 2 && epilogue <= 3, "gemm: bad dtype / layout / epilogue");
  REQ(epilogue != 3 || layout == 1 || dtype == OPTSTAGE_FP32, "gemm: the fp32 store epilogue serves layout 1");
  REQ(M && N && K && M < (1u << 30) && N < (1u << 30) && K < (1u << 30), "gemm: bad extent");
  if (layout == 0) { REQ(lda >= K && ldb >= K, "gemm: leading dimension smaller than K"); }
  else if (layout == 1) { REQ(lda >= M && ldb >= N, "gemm: leading dimension smaller than the row length"); }
  else { REQ(dtype == OPTSTAGE_BF16 && epilogue <= 1 && lda >= K, "gemm: the slab layout serves bf16 store / residual products"); }
  REQ(ldc >= N, "gemm: ldc smaller than N");
  hipError_t e = dtype == OPTSTAGE_BF16
                     ? launch_gemm_bf16(layout, epilogue, A, B, C, R, M, N, K, lda, ldb, ldc, (hipStream_t)stream)
                     : launch_gemm_f32(layout, epilogue, A, B, C, R, M, N, K, lda, ldb, ldc, (hipStream_t)stream);
  return wrap(e, "gemm");
}

optstage_status optstage_op_weight_slabs(const void* src, void* dst, uint32_t N, uint32_t K, uint32_t transposed,
                                         void* stream) {
  REQ(src && dst, "weight_slabs: null operand");
  REQ(N && K && (K % 64) == 0 && N < (1u << 30) && K < (1u << 30) && transposed <= 2, "weight_slabs: bad extent (K must be a multiple of 64)");
  REQ(transposed != 2 || (N % 256) == 0, "weight_slabs: the paired layout needs N = 2 f with f a multiple of 128");
  return wrap(launch_slabs(src, dst, (int)N, (int)K, (int)transposed, (hipStream_t)stream), "weight_slabs");
}

optstage_status optstage_op_gemm_rope(uint32_t layout, const void* A, const void* B, void* C, uint32_t M, uint32_t N,
                                      uint32_t K, uint32_t lda, uint32_t ldb, uint32_t ldc, const float* table, uint32_t seq,
                                      uint32_t rot_cols, void* stream) {
  REQ(A && B && C && table, "gemm_rope: null operand");
  REQ(aligned16(A) && aligned16(B) && aligned16(C) && aligned16(table), "gemm_rope: operands must be 16-byte aligned");
  REQ((layout == 0 || layout == 2) && M && N && K && seq && M < (1u << 30) && N < (1u << 30) && K < (1u << 30), "gemm_rope: bad argument");
  REQ(lda >= K && (layout == 2 || ldb >= K) && ldc >= N, "gemm_rope: leading dimension too small");
  GemmExtra ex;
  ex.table = (const float2*)table; ex.seq = (int)seq; ex.rot_cols = (int)rot_cols;
  return wrap(launch_gemm_bf16((int)layout, EPI_ROPE, A, B, C, nullptr, M, N, K, lda, ldb, ldc, (hipStream_t)stream, &ex), "gemm_rope");
}

optstage_status optstage_op_gemm_swiglu(const void* A, const void* B, void* GU, void* a_out, uint32_t M, uint32_t ffn,
                                        uint32_t K, uint32_t lda, void* stream) {
  REQ(A && B && GU && a_out, "gemm_swiglu: null operand");
  REQ(aligned16(A) && aligned16(B) && aligned16(GU) && aligned16(a_out), "gemm_swiglu: operands must be 16-byte aligned");
  REQ(M && ffn && K && M < (1u << 30) && ffn < (1u << 29) && K < (1u << 30) && lda >= K, "gemm_swiglu: bad argument");
  GemmExtra ex;
  ex.a_out = a_out; ex.f = (int)ffn;
  return wrap(launch_gemm_bf16(GEMM_NT_SLAB, EPI_SWIGLU, A, B, GU, nullptr, M, 2 * ffn, K, lda, 64, 2 * ffn, (hipStream_t)stream, &ex),
              "gemm_swiglu");
}

optstage_status optstage_op_gemm_grouped(uint32_t layout, uint32_t epilogue, uint32_t n,
                                         const optstage_gemm_problem* problems, uint32_t K, void* stream) {
  REQ(problems && n >= 1 && n <= 16 && layout <= 1 && (epilogue == 0 || epilogue == 2 || (epilogue == 3 && layout == 1)),
      "gemm_grouped: bad argument");
  GemmProblem pr[16];
  for (uint32_t i = 0; i < n; ++i) {
    const optstage_gemm_problem& q = problems[i];
    REQ(q.A && q.B && q.C, "gemm_grouped: null operand");
    REQ(aligned16(q.A) && aligned16(q.B) && aligned16(q.C), "gemm_grouped: operands must be 16-byte aligned");
    REQ(q.M && q.N && q.M < (1u << 30) && q.N < (1u << 30) && K && K < (1u << 30), "gemm_grouped: bad extent");
    if (layout == 0) { REQ(q.lda >= K && q.ldb >= K, "gemm_grouped: leading dimension smaller than K"); }
    else { REQ(q.lda >= q.M && q.ldb >= q.N, "gemm_grouped: leading dimension smaller than the row length"); }
    REQ(q.ldc >= q.N, "gemm_grouped: ldc smaller than N");
    pr[i] = {q.A, q.B, q.C, q.R, (int)q.M, (int)q.N, (int)q.lda, (int)q.ldb, (int)q.ldc};
  }
  REQ(gemm_bf16_grouped_applies((int)layout, (int)n, pr, (int)K), "gemm_grouped: the set does not qualify (K % 64, alignment, fewer than 128 tiles)");
  return wrap(launch_gemm_bf16_grouped((int)layout, (int)epilogue, (int)n, pr, (int)K, (hipStream_t)stream), "gemm_grouped");
}

optstage_status optstage_op_norm_fwd(uint32_t dtype, uint32_t family, const void* x, const void* gamma,
                                     const void* beta, void* out, float* stats, uint32_t rows, uint32_t hidden,
                                     float eps, void* stream) {
  REQ(x && gamma && out && stats && (family == OPTSTAGE_LLAMA || beta), "norm_fwd: null operand");
  REQ(dtype <= 1 && family <= 1 && rows && hidden && rows < (1u << 30), "norm_fwd: bad argument");
  return wrap(launch_norm_fwd(dtype, family, x, gamma, beta, out, stats, rows, hidden, eps, (hipStream_t)stream), "norm_fwd");
}

optstage_status optstage_op_norm_bwd(uint32_t dtype, uint32_t family, const void* dn, const void* x,
                                     const float* stats, const void* gamma, const void* dres, void* dx,
                                     float* partial, float* dgamma, float* dbeta, uint32_t rows, uint32_t hidden,
                                     void* stream) {
  REQ(dn && x && stats && gamma && dx && partial && dgamma && (family == OPTSTAGE_LLAMA || dbeta), "norm_bwd: null operand");
  REQ(dtype <= 1 && family <= 1 && rows && hidden && rows < (1u << 30), "norm_bwd: bad argument");
  return wrap(launch_norm_bwd(dtype, family, dn, x, stats, gamma, dres, dx, partial, dgamma, dbeta, rows, hidden, (hipStream_t)stream), "norm_bwd");
}

}  // extern "C"

// Scratch of the entry point that allocates nothing: the per-workgroup gain / bias partials of the norm backward
// kernels, 2 x 256 workgroups x hidden fp32.  One copy per GPU, held until the process ends; host code reaches
// it only through the per-device address resolved below (the symbol's name is not a device address on the host).
namespace {
constexpr uint32_t STATIC_MAX_HIDDEN = 8192;
constexpr int STATIC_PARTIAL_ROWS = 256;
constexpr int STATIC_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) float scratch[2 * STATIC_PARTIAL_ROWS * STATIC_MAX_HIDDEN];
namespace {
std::mutex g_scratch_mu;
float* g_scratch_ptr[STATIC_MAX_DEVICES] = {};

// address of the current device's copy of `scratch`, resolved once per device
optstage_status static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return wrap(e, "norm_bwd_static: hipGetDevice");
  REQ(dev >= 0 && dev < STATIC_MAX_DEVICES, "norm_bwd_static: device index beyond the per-device table");
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return wrap(e, "norm_bwd_static: hipGetSymbolAddress");
    REQ(p, "norm_bwd_static: the scratch symbol resolved to a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return OPTSTAGE_OK;
}
}  // namespace

extern "C" {

optstage_status optstage_op_norm_bwd_static(uint32_t dtype, uint32_t family, const void* dn, const void* x,
                                            const float* stats, const void* gamma, const void* dres, void* dx,
                                            float* dgamma, float* dbeta, uint32_t rows, uint32_t hidden,
                                            void* stream) {
  REQ(dn && x && stats && gamma && dx && dgamma && (family == OPTSTAGE_LLAMA || dbeta), "norm_bwd_static: null operand");
  REQ(dtype <= 1 && family <= 1 && rows && hidden && rows < (1u << 30), "norm_bwd_static: bad argument");
  if (hidden > STATIC_MAX_HIDDEN) {
    char msg[160];
    snprintf(msg, sizeof msg, "norm_bwd_static: hidden %u exceeds the static scratch's maximum of %u", hidden, STATIC_MAX_HIDDEN);
    return (optstage_status)optstage_fail_(OPTSTAGE_E_ARG, msg);
  }
  REQ(norm_bwd_partial_rows((int)rows) <= STATIC_PARTIAL_ROWS, "norm_bwd_static: more partial rows than the static scratch holds");
  float* partial = nullptr;
  optstage_status st = static_scratch(&partial);
  if (st != OPTSTAGE_OK) return st;
  // every partial row the reduction reads is written in full by the first kernel: nothing needs clearing
  return wrap(launch_norm_bwd(dtype, family, dn, x, stats, gamma, dres, dx, partial, dgamma, dbeta, rows, hidden,
      (hipStream_t)stream), "norm_bwd_static");
}

optstage_status optstage_op_act_fwd(uint32_t dtype, uint32_t family, const void* gu, void* a, uint32_t rows,
                                    uint32_t ffn, void* stream) {
  REQ(gu && a && dtype <= 1 && family <= 1 && rows && ffn && rows < (1u << 30) && ffn < (1u << 30), "act_fwd: bad argument");
  return wrap(launch_act_fwd(dtype, family, gu, a, rows, ffn, (hipStream_t)stream), "act_fwd");
}

optstage_status optstage_op_act_bwd(uint32_t dtype, uint32_t family, const void* da, const void* gu, void* dgu,
                                    uint32_t rows, uint32_t ffn, void* stream) {
  REQ(da && gu && dgu && dtype <= 1 && family <= 1 && rows && ffn && rows < (1u << 30) && ffn < (1u << 30), "act_bwd: bad argument");
  return wrap(launch_act_bwd(dtype, family, da, gu, dgu, rows, ffn, (hipStream_t)stream), "act_bwd");
}

optstage_status optstage_op_rope_table(float* table, uint32_t seq, uint32_t head_dim, float base, void* stream) {
  REQ(table && seq && seq < (1u << 24) && head_dim && head_dim <= 1024, "rope_table: bad argument");
  return wrap(launch_rope_table(table, seq, head_dim, base, (hipStream_t)stream), "rope_table");
}

optstage_status optstage_op_rope(uint32_t dtype, const void* src, void* dst, const float* table, uint32_t rows,
                                 uint32_t seq, uint32_t n_q, uint32_t n_kv, uint32_t head_dim, uint32_t backward,
                                 void* stream) {
  REQ(src && dst && table && dtype <= 1 && rows && seq && n_q && n_kv && rows < (1u << 30), "rope: bad argument");
  return wrap(launch_rope(dtype, src, dst, table, rows, seq, n_q, n_kv, head_dim, backward ? 1 : 0, 1, (hipStream_t)stream), "rope");
}

optstage_status optstage_op_attn_fwd(uint32_t dtype, const void* qkv, void* o, float* lse, uint32_t seq,
                                     uint32_t batch, uint32_t n_q, uint32_t n_kv, uint32_t head_dim, void* stream) {
  REQ(qkv && o && lse && dtype <= 1, "attn_fwd: bad argument");
  REQ(seq < (1u << 24) && batch < 65536 && n_q < 65536 && n_kv <= n_q, "attn_fwd: extent out of range");
  return wrap(launch_attn_fwd(dtype, qkv, o, lse, seq, batch, n_q, n_kv, head_dim, (hipStream_t)stream), "attn_fwd");
}

optstage_status optstage_op_attn_bwd(uint32_t dtype, const void* qkv, const void* o, const void* dout,
                                     const float* lse, void* dqkv, float* ws, uint32_t seq, uint32_t batch,
                                     uint32_t n_q, uint32_t n_kv, uint32_t head_dim, void* stream) {
  REQ(qkv && o && dout && lse && dqkv && ws && dtype <= 1 && qkv != dqkv, "attn_bwd: bad argument");
  REQ(seq < (1u << 24) && batch < 65536 && n_q < 65536 && n_kv <= n_q, "attn_bwd: extent out of range");
  return wrap(launch_attn_bwd(dtype, qkv, o, dout, lse, dqkv, ws, seq, batch, n_q, n_kv, head_dim, (hipStream_t)stream), "attn_bwd");
}

uint64_t optstage_op_attn_bwd_ws_floats(uint32_t seq, uint32_t batch, uint32_t n_q, uint32_t n_kv, uint32_t head_dim) {
  return attn_bwd_ws_floats(seq, batch, n_q, n_kv, head_dim);
}

optstage_status optstage_op_checksum(const void* buf, uint64_t bytes, uint64_t* out_dev, void* stream) {
  REQ(buf && out_dev && ((uintptr_t)buf & 7) == 0, "checksum: bad argument");
  return wrap(launch_checksum(buf, bytes, out_dev, (hipStream_t)stream), "checksum");
}

}  // extern "C"
