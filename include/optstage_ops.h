/*
 * Single-kernel entry points of liboptstage: each launches one step of a stage's F / B / W op graph
 * (paper Sec. 2.2: linear maps z = W x, grad_x = W^T grad_z, grad_W = grad_z x^T; everything else is the
 * non-linear part the paper folds into sigma).  They exist so that every kernel can be checked against
 * the CPU oracle and timed on its own; the stage calls in optstage.h launch exactly these kernels.
 *
 * All tensor pointers are DEVICE memory, caller-owned, 16-byte aligned, row-major with tokens as rows.
 * dtype is optstage_dtype (storage type; arithmetic is fp32 / bf16 MFMA with fp32 accumulation).
 * stream is a hipStream_t.  Calls only enqueue; errors are reported as optstage_status with a message
 * in optstage_last_error().  Shapes the kernels cannot handle are rejected on the host (OPTSTAGE_E_ARG), and so
 * is a null pointer or an extent of zero: a refused call launches nothing and writes nothing.
 */
#ifndef OPTSTAGE_OPS_H
#define OPTSTAGE_OPS_H

#include "optstage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = sum_k A(m,k) B(n,k).
 * layout 0 (NT): A is [M,K] (lda), B is [N,K] (ldb)  -- forward Y = X W^T and dX = dY (W^T)^T
 * layout 1 (TN): A is [K,M] (lda), B is [K,N] (ldb)  -- dW = dY^T X
 * layout 2 (NT, B in slabs; bf16, epilogue 0 or 1): A as in layout 0; B(n,k) at element offset
 *          ((n / 256) * (K / 64) + k / 64) * 16384 + (n % 256) * 64 + k % 64, i.e. the 256 rows x 64 columns that one
 *          workgroup loads per step of the contraction are consecutive in memory (how the stage keeps its weight
 *          copies); B spans ceil(N / 256) * (K / 64) slabs, rows past N are never used; ldb is ignored.  Needs
 *          K % 64 == 0 and at least 128 output tiles of 256 x 256, else OPTSTAGE_E_ARG.
 * epilogue 0: C (stage dtype) = product; 1: C = product + R (R like C); 2: C (fp32) += product;
 *          3: C (fp32) = product (layout 1 only for bf16: the first weight-gradient product of an iteration).
 * bf16 needs lda, ldb multiples of 8, N and ldc multiples of 4, K (NT) or M and N (TN) multiples of 8. */
optstage_status optstage_op_gemm(uint32_t dtype, uint32_t layout, uint32_t epilogue, const void* A, const void* B,
                                 void* C, const void* R, uint32_t M, uint32_t N, uint32_t K, uint32_t lda,
                                 uint32_t ldb, uint32_t ldc, void* stream);

/* Writes a bf16 matrix into the slab layout of layout 2: dst (DEVICE, ceil(N / 256) * 256 * K elements) receives
 * B(n,k) = src[n * K + k] (transposed = 0) or src[k * N + n] (transposed = 1: the source is [K,N]); rows past N are
 * zero.  K % 64 must be 0.  transposed = 2 (paired, for optstage_op_gemm_swiglu): src is a [gate | up] weight of N = 2 f
 * rows [N,K], f % 128 == 0, and slab row 256 t + 128 w + 64 q + o holds source row q f + 128 t + 64 w + o (q = 0 gate,
 * 1 up), so that every 128-column half of an output tile is 64 gate columns beside the 64 matching up columns.  The
 * stage does this for its weight copies in optstage_set_weight. */
optstage_status optstage_op_weight_slabs(const void* src, void* dst, uint32_t N, uint32_t K, uint32_t transposed,
                                         void* stream);

/* The QKV projection with the rotary embedding fused into its epilogue (bf16): C = A B^T as optstage_op_gemm with
 * layout 0 or 2, then, before the one rounding to bf16, the first rot_cols columns (the q and k heads, a multiple of
 * 128; head_dim is 128) are rotated by position = row % seq with the pairing and the table of optstage_op_rope.  Needs
 * N % 128 == 0 and a shape the direct kernel serves (K % 64 == 0, at least 128 output tiles of 256 x 256), else
 * OPTSTAGE_E_ARG.  Same result as optstage_op_gemm followed by optstage_op_rope except for that one rounding less. */
optstage_status optstage_op_gemm_rope(uint32_t layout, const void* A, const void* B, void* C, uint32_t M, uint32_t N,
                                      uint32_t K, uint32_t lda, uint32_t ldb, uint32_t ldc, const float* table, uint32_t seq,
                                      uint32_t rot_cols, void* stream);
/* The gate / up projection with the MLP activation fused into its epilogue (bf16, LLAMA): B is the [gate | up] weight
 * [2 ffn, K] in PAIRED slabs (optstage_op_weight_slabs with transposed = 2).  Writes GU [M, 2 ffn] = A B^T in the plain
 * [gate | up] layout (what the backward pass reads) and a_out [M, ffn] = silu(gate) * up formed from the fp32
 * accumulators.  ffn % 128 == 0, K % 64 == 0 and at least 128 output tiles, else OPTSTAGE_E_ARG. */
optstage_status optstage_op_gemm_swiglu(const void* A, const void* B, void* GU, void* a_out, uint32_t M, uint32_t ffn,
                                        uint32_t K, uint32_t lda, void* stream);

/* n (1..16) independent bf16 products of the same layout, epilogue and K in ONE launch (the weight-gradient GEMMs
 * of a W op, dW = dY^T X for every linear of every layer, do not depend on one another: Sec. 2.2).  problems is a
 * HOST array; pointers inside are DEVICE.  Each problem must satisfy optstage_op_gemm's alignment rules, K % 64
 * must be 0 and the set must hold at least 128 tiles of 256 x 256; otherwise OPTSTAGE_E_ARG and nothing runs. */
typedef struct { const void* A; const void* B; void* C; const void* R; uint32_t M, N, lda, ldb, ldc; } optstage_gemm_problem;
optstage_status optstage_op_gemm_grouped(uint32_t layout, uint32_t epilogue, uint32_t n,
                                         const optstage_gemm_problem* problems, uint32_t K, void* stream);

/* family LLAMA: RMSNorm, stats[rows] = rstd.  family GPT: LayerNorm, stats[2*row] = mean, [2*row+1] = rstd. */
optstage_status optstage_op_norm_fwd(uint32_t dtype, uint32_t family, const void* x, const void* gamma,
                                     const void* beta, void* out, float* stats, uint32_t rows, uint32_t hidden,
                                     float eps, void* stream);
/* dx = (dres ? dres : 0) + norm'(dn); dgamma (and dbeta for GPT) fp32 [hidden] are ADDED to.
 * partial: fp32 scratch of 2 * min(rows, 512) * hidden elements. */
optstage_status optstage_op_norm_bwd(uint32_t dtype, uint32_t family, const void* dn, const void* x,
                                     const float* stats, const void* gamma, const void* dres, void* dx,
                                     float* partial, float* dgamma, float* dbeta, uint32_t rows, uint32_t hidden,
                                     void* stream);
/* optstage_op_norm_bwd for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without `partial`, same kernels,
 * bit-identical results.  The partials live in a 16 MiB array that is part of the library's device image (one copy
 * per GPU, held until the process ends); the call allocates nothing and frees nothing.  hidden may be at most 8192,
 * else OPTSTAGE_E_ARG and nothing runs.  All calls on one GPU share that array: two calls that overlap in time on
 * one GPU (different streams, or different host threads) race; calls on one stream are safe.  The first call on a
 * device resolves the array's address there (a HIP runtime call that may load the code object). */
optstage_status optstage_op_norm_bwd_static(uint32_t dtype, uint32_t family, const void* dn, const void* x,
                                            const float* stats, const void* gamma, const void* dres, void* dx,
                                            float* dgamma, float* dbeta, uint32_t rows, uint32_t hidden,
                                            void* stream);
/* LLAMA: a[rows, f] = silu(gu[:, :f]) * gu[:, f:], gu is [rows, 2f].  GPT: a = gelu(gu), gu is [rows, f]. */
optstage_status optstage_op_act_fwd(uint32_t dtype, uint32_t family, const void* gu, void* a, uint32_t rows,
                                    uint32_t ffn, void* stream);
/* dgu like gu; dgu may alias gu. */
optstage_status optstage_op_act_bwd(uint32_t dtype, uint32_t family, const void* da, const void* gu, void* dgu,
                                    uint32_t rows, uint32_t ffn, void* stream);
/* table: fp32 [seq][head_dim/2][2] = (cos, sin)(pos * base^(-2k/head_dim)). */
optstage_status optstage_op_rope_table(float* table, uint32_t seq, uint32_t head_dim, float base, void* stream);
/* Rotates the q and k heads of packed qkv rows [rows, (n_q + 2 n_kv) * head_dim], position = row % seq,
 * pairing element k with k + head_dim/2.  backward != 0 applies the transposed rotation.  dst may be src
 * (in place); otherwise the v part is copied too. */
optstage_status optstage_op_rope(uint32_t dtype, const void* src, void* dst, const float* table, uint32_t rows,
                                 uint32_t seq, uint32_t n_q, uint32_t n_kv, uint32_t head_dim, uint32_t backward,
                                 void* stream);
/* Causal attention over packed qkv [batch*seq, (n_q + 2 n_kv) * d]; q-head a reads kv-head a*n_kv/n_q.
 * o is [batch*seq, n_q*d]; lse fp32 [batch][n_q][seq] (natural log). head_dim 64 or 128. */
optstage_status optstage_op_attn_fwd(uint32_t dtype, const void* qkv, void* o, float* lse, uint32_t seq,
                                     uint32_t batch, uint32_t n_q, uint32_t n_kv, uint32_t head_dim, void* stream);
/* dqkv like qkv (must not alias it).  ws: fp32 scratch of optstage_op_attn_bwd_ws_floats() elements. */
optstage_status optstage_op_attn_bwd(uint32_t dtype, const void* qkv, const void* o, const void* dout,
                                     const float* lse, void* dqkv, float* ws, uint32_t seq, uint32_t batch,
                                     uint32_t n_q, uint32_t n_kv, uint32_t head_dim, void* stream);
uint64_t optstage_op_attn_bwd_ws_floats(uint32_t seq, uint32_t batch, uint32_t n_q, uint32_t n_kv, uint32_t head_dim);
/* out_dev[0] = sum of the buffer's 64-bit words mod 2^64, out_dev[1] = their xor.  bytes % 8 == 0. */
optstage_status optstage_op_checksum(const void* buf, uint64_t bytes, uint64_t* out_dev, void* stream);

/* Pure host, no GPU needed: runs the ordering rules and the list-order memory accounting (Eq. 6, Eq. 7,
 * fixed micro-batch order, offload / reload rules) over a whole list for the stage described by desc
 * (shape fields, n_microbatches and hbm_budget_bytes are read; 0 budget = unlimited).  *peak_bytes is the
 * highest live byte count reached (up to the failing event on error); live_after (may be null, HOST,
 * n entries) receives the live bytes after each event. */
optstage_status optstage_plan(const optstage_desc* desc, const optstage_event* events, size_t n, size_t* first_bad,
                              uint64_t* peak_bytes, uint64_t* live_after);

#ifdef __cplusplus
}
#endif
#endif
