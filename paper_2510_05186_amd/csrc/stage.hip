// Stage runtime: memory table, list-order activation accounting under the HBM budget (Eq. 7), the
// physical arena, the offload / reload engine (side stream + events, Eq. 12-14) and the executor that
// walks a per-stage event list and enqueues the F / B / W op graphs (Sec. 2.2, Sec. 3).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/optstage.h"
#include "../../include/optstage_ops.h"
#include "arena.h"
#include "common.h"

namespace {

thread_local char g_err[512] = "";

optstage_status fail(optstage_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}
}  // namespace

// used by the single-op wrappers in ops.hip
int optstage_fail_(int status, const char* msg) {
  snprintf(g_err, sizeof g_err, "%s", msg);
  return status;
}

namespace {

#define HIP_TRY(expr)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess) return fail(OPTSTAGE_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr uint64_t ALIGN = 256;
constexpr int NK = OPTSTAGE_N_KINDS;
constexpr int NFK = OPTSTAGE_N_F_KINDS;
// kinds that are cheap functions of kinds F keeps anyway (norm outputs, MLP activation output)
inline bool recomputable(int k) { return k == OPTSTAGE_K_N1 || k == OPTSTAGE_K_N2 || k == OPTSTAGE_K_A; }
uint64_t round_up(uint64_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }

struct Shape {
  int family, dtype, L, h, nq, nkv, d, f, seq, mb, tokens, qkv_w, up_w, e;
  int chunks, Lc;   // model chunks on this stage and layers per chunk (L = chunks * Lc)
  bool fuse_rope, fuse_act;   // rotary in the QKV projection's epilogue, MLP activation in the gate / up projection's
};

optstage_status shape_from_desc(const optstage_desc* d, Shape* s) {
  if (!d) return fail(OPTSTAGE_E_ARG, "desc is null");
  if (d->struct_size != sizeof(optstage_desc)) return fail(OPTSTAGE_E_ARG, "desc.struct_size mismatch");
  if (d->family > 1 || d->dtype > 1 || d->recompute > 1 || d->no_fusion > 1 || d->reserved)
    return fail(OPTSTAGE_E_ARG, "bad family, dtype, recompute or no_fusion");
  if (!d->n_layers || !d->hidden || !d->n_q_heads || !d->n_kv_heads || !d->ffn || !d->seq || !d->micro_batch || !d->n_microbatches)
    return fail(OPTSTAGE_E_ARG, "zero-sized shape field");
  if (d->head_dim != 64 && d->head_dim != 128) return fail(OPTSTAGE_E_ARG, "head_dim must be 64 or 128");
  if (d->n_q_heads % d->n_kv_heads) return fail(OPTSTAGE_E_ARG, "n_q_heads must be a multiple of n_kv_heads");
  const int vec = d->dtype == OPTSTAGE_BF16 ? 8 : 4;
  if (d->hidden % vec || d->ffn % vec) return fail(OPTSTAGE_E_ARG, "hidden and ffn must be multiples of %d", vec);
  if (d->hidden / vec > 1024) return fail(OPTSTAGE_E_ARG, "hidden too large for the norm kernels");
  if ((uint64_t)d->seq * d->micro_batch > (1u << 24)) return fail(OPTSTAGE_E_ARG, "too many tokens per micro-batch");
  s->family = d->family; s->dtype = d->dtype; s->L = d->n_layers; s->h = d->hidden; s->nq = d->n_q_heads;
  s->nkv = d->n_kv_heads; s->d = d->head_dim; s->f = d->ffn; s->seq = d->seq; s->mb = d->micro_batch;
  s->tokens = d->seq * d->micro_batch;
  s->qkv_w = (s->nq + 2 * s->nkv) * s->d;
  s->up_w = s->family == OPTSTAGE_LLAMA ? 2 * s->f : s->f;
  s->e = s->dtype == OPTSTAGE_BF16 ? 2 : 4;
  s->chunks = d->n_chunks ? (int)d->n_chunks : 1;
  if (s->L % s->chunks) return fail(OPTSTAGE_E_ARG, "n_layers must be a multiple of n_chunks");
  s->Lc = s->L / s->chunks;
  const bool fusable = !d->no_fusion && s->family == OPTSTAGE_LLAMA && s->dtype == OPTSTAGE_BF16;
  s->fuse_rope = fusable && gemm_bf16_fused_applies(EPI_ROPE, s->tokens, s->qkv_w, s->h, s->h, s->d);
  // not in the recompute variant: B rebuilds the activation output from the stored gate / up tensor and has to arrive
  // at the very bits F multiplied with
  s->fuse_act = fusable && !d->recompute && (s->f % 128) == 0 && gemm_bf16_fused_applies(EPI_SWIGLU, s->tokens, s->up_w, s->h, s->h, 0);
  return OPTSTAGE_OK;
}

// exact (unpadded) byte size of each activation kind for one layer of one micro-batch
void kind_raw_bytes(const Shape& s, uint64_t raw[NK]) {
  const uint64_t t = s.tokens, e = s.e;
  raw[OPTSTAGE_K_X_IN] = t * s.h * e;
  raw[OPTSTAGE_K_N1] = t * s.h * e;
  raw[OPTSTAGE_K_QKV] = t * s.qkv_w * e;
  raw[OPTSTAGE_K_O] = t * s.nq * s.d * e;
  raw[OPTSTAGE_K_LSE] = (uint64_t)s.nq * t * 4;
  raw[OPTSTAGE_K_X_MID] = t * s.h * e;
  raw[OPTSTAGE_K_N2] = t * s.h * e;
  raw[OPTSTAGE_K_GU] = t * s.up_w * e;
  raw[OPTSTAGE_K_A] = t * s.f * e;
  raw[OPTSTAGE_K_STATS] = (s.family == OPTSTAGE_LLAMA ? 2 : 4) * t * 4;
  raw[OPTSTAGE_K_DY] = t * s.h * e;
  raw[OPTSTAGE_K_DX_MID] = t * s.h * e;
}

struct WorkspaceLayout {
  uint64_t rope, wt_base, wt[OPTSTAGE_N_WEIGHTS], wf[OPTSTAGE_N_WEIGHTS], wt_layer_stride, da, dn, dout, dqkv, attn, partial,
      csum, total;
};

uint64_t weight_elems(const Shape& s, int which) {
  switch (which) {
    case OPTSTAGE_W_QKV: return (uint64_t)s.qkv_w * s.h;
    case OPTSTAGE_W_O: return (uint64_t)s.h * s.nq * s.d;
    case OPTSTAGE_W_GU: return (uint64_t)s.up_w * s.h;
    case OPTSTAGE_W_D: return (uint64_t)s.h * s.f;
    default: return s.h;
  }
}

// rows (outputs) and columns (inputs) of a linear weight; false for the norm parameters
bool weight_dims(const Shape& s, int which, int* rows, int* cols) {
  switch (which) {
    case OPTSTAGE_W_QKV: *rows = s.qkv_w; *cols = s.h; return true;
    case OPTSTAGE_W_O: *rows = s.h; *cols = s.nq * s.d; return true;
    case OPTSTAGE_W_GU: *rows = s.up_w; *cols = s.h; return true;
    case OPTSTAGE_W_D: *rows = s.h; *cols = s.f; return true;
    default: return false;
  }
}

// Which of a weight's two GEMM operand copies are kept in the slab layout (256 rows x 64 columns per slab, what a
// workgroup of the direct bf16 kernel loads per k-tile, consecutive in memory): the forward operand W (y = x W^T)
// and the transposed one (dx = dy W).  A shape the direct kernel does not serve keeps the plain copies.
void slab_modes(const Shape& s, int which, bool* fwd, bool* bwd) {
  int rows = 0, cols = 0;
  *fwd = *bwd = false;
  if (s.dtype != OPTSTAGE_BF16 || !weight_dims(s, which, &rows, &cols)) return;
  *fwd = gemm_bf16_slab_applies(s.tokens, rows, cols, cols);
  *bwd = gemm_bf16_slab_applies(s.tokens, cols, rows, rows);
}

WorkspaceLayout workspace_layout(const Shape& s) {
  WorkspaceLayout w;
  memset(&w, 0, sizeof w);
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += round_up(bytes); return o; };
  w.rope = take(s.family == OPTSTAGE_LLAMA ? (uint64_t)s.seq * (s.d / 2) * 8 : 0);
  uint64_t lstart = off;
  w.wt_base = lstart;
  for (int k : {OPTSTAGE_W_QKV, OPTSTAGE_W_O, OPTSTAGE_W_GU, OPTSTAGE_W_D}) {
    int rows = 0, cols = 0;
    bool sf, sb;
    weight_dims(s, k, &rows, &cols);
    slab_modes(s, k, &sf, &sb);
    // transposed copy [cols][rows] (slabs pad its rows to a multiple of 256); forward slab copy only where it is used
    w.wt[k] = take((uint64_t)(sb ? (cols + 255) / 256 * 256 : cols) * rows * s.e) - lstart;
    w.wf[k] = take(sf ? (uint64_t)((rows + 255) / 256 * 256) * cols * s.e : 0) - lstart;
  }
  w.wt_layer_stride = off - lstart;
  off = lstart + w.wt_layer_stride * s.L;
  w.da = take((uint64_t)s.tokens * s.f * s.e);
  w.dn = take((uint64_t)s.tokens * s.h * s.e);
  w.dout = take((uint64_t)s.tokens * s.nq * s.d * s.e);
  w.dqkv = take((uint64_t)s.tokens * s.qkv_w * s.e);
  w.attn = take(attn_bwd_ws_floats(s.seq, s.mb, s.nq, s.nkv, s.d) * 4);
  w.partial = take((uint64_t)2 * norm_bwd_partial_rows(s.tokens) * s.h * 4);
  w.csum = take(16);
  w.total = off;
  return w;
}

enum BufState : uint8_t { B_NONE = 0, B_DEV, B_OFFLOADING, B_HOST, B_RELOADED };

struct BufRec {
  uint8_t state = B_NONE;
  uint64_t dev_off = 0, host_off = 0;
};

struct MbState {
  bool f = false, b = false, w = false;
};

// Pure host, copyable: everything the validator needs.
struct Logical {
  int L = 0, m = 0, chunks = 1, Lc = 0;
  bool recompute = false;   // F keeps no N1 / N2 / A; B rebuilds them for W
  uint64_t bytes[NK] = {}, budget = 0, live = 0, peak = 0;
  std::vector<int> next_f, next_b, next_w;   // [chunk]
  std::vector<MbState> mbs;                  // [chunk][mb]
  std::vector<BufRec> bufs;   // [mb][layer][kind]
  BlockArena arena, host;
  BufRec& buf(int j, int l, int k) { return bufs[((size_t)j * L + l) * NK + k]; }
};

struct OpBufs {   // device offsets an op touches, captured before its releases; host offsets for O / R
  std::vector<uint64_t> dev, host;   // [layer][kind]
};

// op >= 0: schedule op; op < 0: kernel class -(op + 1); op == SPAN_STALL: the compute stream waiting for transfers.
// trace >= 0: the entry of the executed trace that receives the span's times
constexpr int SPAN_STALL = 100;
struct TimedSpan { int op; hipEvent_t a, b; int trace; };

}  // namespace

struct optstage {
  optstage_desc desc;
  Shape sh;
  WorkspaceLayout ws;
  uint64_t raw[NK];
  Logical lg;
  hipStream_t cs, xs, rs;   // compute, copy (offloads), reloads (= xs unless the caller gave a stream of its own)
  std::vector<const void*> w;          // [layer][which]
  std::vector<float*> gw;              // [layer][which]
  std::vector<const void*> x_in, dy_out;
  std::vector<void*> y_out, dx_in;
  std::vector<hipEvent_t> ev_f, ev_o, ev_r, ev_pos;   // [mb], [mb][layer] x3
  std::vector<hipEvent_t> ev_fl;                      // [mb][layer]: that layer's forward kernels of F mb have ended
  hipEvent_t last_r = nullptr;   // event of the most recent reload (separate reload stream only)
  std::vector<hipEvent_t> tpool;
  size_t tnext = 0;
  std::vector<TimedSpan> spans;
  optstage_stats stats;
  bool ktiming = false;
  bool failed = false;           // a HIP call failed while a list was being enqueued: unusable until optstage_reset
  bool overwrite = false;        // the first B / W of an iteration store the gradients instead of adding to them
  hipEvent_t origin = nullptr;   // recorded on the compute stream when the first event after a reset is enqueued
  bool origin_set = false;
  std::vector<optstage_trace_entry> trace;   // executed events since the last reset
  std::vector<uint8_t> reloaded;             // [chunk][mb]: a reload of this micro-batch was enqueued this iteration
  uint64_t in_flight = 0, min_live = UINT64_MAX;
  double sum_live = 0.0;
  char* arena() const { return (char*)desc.arena; }
  char* wsp() const { return (char*)desc.workspace; }
};

namespace {

optstage_status alloc_dev(Logical& lg, int j, int l, int k) {
  BufRec& b = lg.buf(j, l, k);
  const uint64_t n = lg.bytes[k];
  if (lg.budget && lg.live + n > lg.budget)
    return fail(OPTSTAGE_E_BUDGET, "micro-batch %d layer %d kind %d needs %llu live bytes, budget %llu", j, l, k,
                (unsigned long long)(lg.live + n), (unsigned long long)lg.budget);
  uint64_t off = lg.arena.alloc(n);
  if (off == UINT64_MAX)
    return fail(OPTSTAGE_E_ARENA, "arena cannot place %llu bytes (largest free range %llu of %llu)", (unsigned long long)n,
                (unsigned long long)lg.arena.largest_free(), (unsigned long long)lg.arena.capacity());
  b.dev_off = off;
  lg.live += n;
  if (lg.live > lg.peak) lg.peak = lg.live;
  return OPTSTAGE_OK;
}

void free_dev(Logical& lg, int j, int l, int k) {
  BufRec& b = lg.buf(j, l, k);
  lg.arena.release(b.dev_off, lg.bytes[k]);
  lg.live -= lg.bytes[k];
}

// Applies one event to the logical state.  On error the state may be partly modified: callers run it
// on a scratch copy first.
optstage_status apply_event(Logical& lg, const optstage_event& ev, OpBufs* out) {
  const int L = lg.L;
  const int j = (int)ev.microbatch;
  if (ev.microbatch >= (uint32_t)lg.m) return fail(OPTSTAGE_E_ARG, "micro-batch %u out of range", ev.microbatch);
  if (out) { out->dev.assign((size_t)L * NK, UINT64_MAX); out->host.assign((size_t)L * NK, UINT64_MAX); }
  auto note = [&](int l, int k) { if (out) out->dev[(size_t)l * NK + k] = lg.buf(j, l, k).dev_off; };
  // F / B / W: the event's layer field is the model chunk; O / OWAIT / R: the chunk that holds the layer
  const bool compute = ev.op <= OPTSTAGE_W;
  if (compute && ev.layer >= (uint32_t)lg.chunks) return fail(OPTSTAGE_E_ARG, "chunk %u out of range", ev.layer);
  if (!compute && ev.op <= OPTSTAGE_R && ev.layer >= (uint32_t)L) return fail(OPTSTAGE_E_ARG, "layer %u out of range", ev.layer);
  const int c = compute ? (int)ev.layer : (ev.op <= OPTSTAGE_R ? (int)ev.layer / lg.Lc : 0);
  const int l0 = c * lg.Lc, l1 = l0 + lg.Lc;      // the chunk's layers
  MbState& mb = lg.mbs[(size_t)c * lg.m + j];
  optstage_status st;
  switch (ev.op) {
    case OPTSTAGE_F: {
      if (mb.f) return fail(OPTSTAGE_E_ORDER, "F %d listed twice", j);
      if (j != lg.next_f[c]) return fail(OPTSTAGE_E_ORDER, "F ops must run in increasing micro-batch order (expected %d, got %d)", lg.next_f[c], j);
      for (int l = l0; l < l1; ++l)
        for (int k = 0; k < NFK; ++k) {
          if (lg.recompute && recomputable(k)) continue;
          if ((st = alloc_dev(lg, j, l, k)) != OPTSTAGE_OK) return st;
          lg.buf(j, l, k).state = B_DEV;
          note(l, k);
        }
      mb.f = true;
      lg.next_f[c]++;
      return OPTSTAGE_OK;
    }
    case OPTSTAGE_B: {
      if (mb.b) return fail(OPTSTAGE_E_ORDER, "B %d listed twice", j);
      if (!mb.f) return fail(OPTSTAGE_E_ORDER, "B %d before F %d", j, j);
      if (j != lg.next_b[c]) return fail(OPTSTAGE_E_ORDER, "B ops must run in increasing micro-batch order (expected %d, got %d)", lg.next_b[c], j);
      for (int l = l0; l < l1; ++l)
        for (int k = 0; k < NFK; ++k) {
          if (lg.recompute && recomputable(k)) continue;
          uint8_t s = lg.buf(j, l, k).state;
          if (s != B_DEV && s != B_RELOADED)
            return fail(OPTSTAGE_E_ORDER, "B %d while layer %d kind %d is offloaded and not reloaded", j, l, k);
          note(l, k);
        }
      auto make = [&](int l, int k) -> optstage_status {
        optstage_status s2 = alloc_dev(lg, j, l, k);
        if (s2 == OPTSTAGE_OK) { lg.buf(j, l, k).state = B_DEV; note(l, k); }
        return s2;
      };
      auto drop = [&](int l, int k) { free_dev(lg, j, l, k); lg.buf(j, l, k).state = B_NONE; };
      if ((st = make(l1 - 1, OPTSTAGE_K_DY)) != OPTSTAGE_OK) return st;
      // every buffer is made before the kernel that first writes it and dropped after its last reader, in the
      // order B enqueues its kernels: a region released here may be handed out again within the same op
      for (int l = l1 - 1; l >= l0; --l) {
        if (lg.recompute) {
          if ((st = make(l, OPTSTAGE_K_A)) != OPTSTAGE_OK) return st;
          if ((st = make(l, OPTSTAGE_K_N2)) != OPTSTAGE_OK) return st;
        }
        if ((st = make(l, OPTSTAGE_K_DX_MID)) != OPTSTAGE_OK) return st;
        drop(l, OPTSTAGE_K_X_MID);
        drop(l, OPTSTAGE_K_LSE);
        if (lg.recompute && (st = make(l, OPTSTAGE_K_N1)) != OPTSTAGE_OK) return st;
        if (l > l0 && (st = make(l - 1, OPTSTAGE_K_DY)) != OPTSTAGE_OK) return st;
        drop(l, OPTSTAGE_K_X_IN);
        drop(l, OPTSTAGE_K_STATS);
      }
      mb.b = true;
      lg.next_b[c]++;
      return OPTSTAGE_OK;
    }
    case OPTSTAGE_W: {
      if (mb.w) return fail(OPTSTAGE_E_ORDER, "W %d listed twice", j);
      if (!mb.b) return fail(OPTSTAGE_E_ORDER, "W %d before B %d", j, j);
      if (j != lg.next_w[c]) return fail(OPTSTAGE_E_ORDER, "W ops must run in increasing micro-batch order (expected %d, got %d)", lg.next_w[c], j);
      static const int freed[] = {OPTSTAGE_K_N1, OPTSTAGE_K_QKV, OPTSTAGE_K_O, OPTSTAGE_K_DX_MID,
                                  OPTSTAGE_K_N2, OPTSTAGE_K_GU, OPTSTAGE_K_A, OPTSTAGE_K_DY};
      for (int l = l0; l < l1; ++l)
        for (int k : freed) {
          note(l, k);
          free_dev(lg, j, l, k);
          lg.buf(j, l, k).state = B_NONE;
        }
      mb.w = true;
      lg.next_w[c]++;
      return OPTSTAGE_OK;
    }
    case OPTSTAGE_O:
    case OPTSTAGE_OWAIT:
    case OPTSTAGE_R: {
      if (!ev.kind_mask || (ev.kind_mask >> NFK)) return fail(OPTSTAGE_E_ARG,
          "kind_mask 0x%x names no offloadable kind or a non-offloadable one", ev.kind_mask);
      const int l = (int)ev.layer;
      for (int k = 0; k < NFK; ++k) {
        if (!(ev.kind_mask & (1u << k))) continue;
        BufRec& b = lg.buf(j, l, k);
        if (ev.op == OPTSTAGE_O) {
          if (!mb.f || mb.b) return fail(OPTSTAGE_E_ORDER, "offload of micro-batch %d outside its F..B window", j);
          if (b.state != B_DEV) return fail(OPTSTAGE_E_ORDER,
              "offload of micro-batch %d layer %d kind %d: not resident or already offloaded", j, l, k);
          uint64_t ho = lg.host.alloc(lg.bytes[k]);
          if (ho == UINT64_MAX) return fail(OPTSTAGE_E_HOSTPOOL, "pinned host pool exhausted (%llu bytes)", (unsigned long long)lg.host.capacity());
          b.host_off = ho;
          b.state = B_OFFLOADING;
        } else if (ev.op == OPTSTAGE_OWAIT) {
          if (b.state != B_OFFLOADING) return fail(OPTSTAGE_E_ORDER, "OWAIT of micro-batch %d layer %d kind %d without a pending offload", j, l, k);
          note(l, k);
          free_dev(lg, j, l, k);
          b.state = B_HOST;
        } else {
          if (b.state != B_HOST) return fail(OPTSTAGE_E_ORDER, "reload of micro-batch %d layer %d kind %d before its offload completed", j, l, k);
          if ((st = alloc_dev(lg, j, l, k)) != OPTSTAGE_OK) return st;
          lg.host.release(b.host_off, lg.bytes[k]);
          b.state = B_RELOADED;
        }
        if (out) {
          out->dev[(size_t)l * NK + k] = b.dev_off;
          out->host[(size_t)l * NK + k] = b.host_off;
        }
      }
      return OPTSTAGE_OK;
    }
    default:
      return fail(OPTSTAGE_E_ARG, "unknown op %u", ev.op);
  }
}

optstage_status check_complete(const Logical& lg) {
  for (size_t i = 0; i < lg.mbs.size(); ++i)
    if (!lg.mbs[i].f || !lg.mbs[i].b || !lg.mbs[i].w)
      return fail(OPTSTAGE_E_ORDER, "micro-batch %d of chunk %d is missing F, B or W", (int)(i % lg.m), (int)(i / lg.m));
  return OPTSTAGE_OK;
}

hipError_t gemm(const Shape& s, int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                int K, int lda, int ldb, int ldc, hipStream_t st) {
  return s.dtype == OPTSTAGE_BF16 ? launch_gemm_bf16(layout, epi, A, B, C, R, M, N, K, lda, ldb, ldc, st)
                                  : launch_gemm_f32(layout, epi, A, B, C, R, M, N, K, lda, ldb, ldc, st);
}

hipEvent_t timing_event(optstage* st) {
  if (st->tnext == st->tpool.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    st->tpool.push_back(e);
  }
  return st->tpool[st->tnext++];
}

optstage_status span_begin(optstage* st, int op, hipStream_t s, TimedSpan* sp, int trace = -1) {
  sp->op = op;
  sp->trace = trace;
  sp->a = timing_event(st);
  sp->b = timing_event(st);
  if (!sp->a || !sp->b) return fail(OPTSTAGE_E_HIP, "hipEventCreate failed");
  HIP_TRY(hipEventRecord(sp->a, s));
  return OPTSTAGE_OK;
}
optstage_status span_end(optstage* st, hipStream_t s, const TimedSpan& sp) {
  HIP_TRY(hipEventRecord(sp.b, s));
  st->spans.push_back(sp);
  return OPTSTAGE_OK;
}

// optional per-kernel timing: brackets one launch with events and books its algorithmic work
#define KT(cls, work, call)                                                   \
  do {                                                                        \
    TimedSpan ksp_;                                                           \
    if (st->ktiming) {                                                        \
      optstage_status r_ = span_begin(st, -(int)(cls) - 1, st->cs, &ksp_);    \
      if (r_ != OPTSTAGE_OK) return r_;                                       \
    }                                                                         \
    HIP_TRY(call);                                                            \
    if (st->ktiming) {                                                        \
      optstage_status r_ = span_end(st, st->cs, ksp_);                        \
      if (r_ != OPTSTAGE_OK) return r_;                                       \
      st->stats.kernel_launches[cls]++;                                       \
      st->stats.kernel_work[cls] += (double)(work);                           \
    }                                                                         \
  } while (0)

const void* W(optstage* st, int l, int which) { return st->w[(size_t)l * OPTSTAGE_N_WEIGHTS + which]; }
float* GW(optstage* st, int l, int which) { return st->gw[(size_t)l * OPTSTAGE_N_WEIGHTS + which]; }
const void* WT(optstage* st, int l, int which) { return st->wsp() + st->ws.wt_base + st->ws.wt_layer_stride * l + st->ws.wt[which]; }
const void* WF(optstage* st, int l, int which) { return st->wsp() + st->ws.wt_base + st->ws.wt_layer_stride * l + st->ws.wf[which]; }
// B operand and layout code of the forward (y = x W^T) and backward (dx = dy W) GEMM of a weight
const void* fwd_operand(optstage* st, int l, int which, int* layout) {
  bool sf, sb;
  slab_modes(st->sh, which, &sf, &sb);
  *layout = sf ? GEMM_NT_SLAB : GEMM_NT;
  return sf ? WF(st, l, which) : W(st, l, which);
}
const void* bwd_operand(optstage* st, int l, int which, int* layout) {
  bool sf, sb;
  slab_modes(st->sh, which, &sf, &sb);
  *layout = sb ? GEMM_NT_SLAB : GEMM_NT;
  return WT(st, l, which);
}


#define TRY(x)                               \
  do {                                       \
    optstage_status t_ = (x);                \
    if (t_ != OPTSTAGE_OK) return t_;        \
  } while (0)

optstage_status k_gemm(optstage* st, int layout, int epi, const void* A, const void* B, void* C, const void* R, int M,
                       int N, int K, int lda, int ldb, int ldc, int cls = -1) {
  if (cls < 0) cls = layout == GEMM_TN ? OPTSTAGE_KC_GEMM_TN_ACCUM : (epi == EPI_RESID ? OPTSTAGE_KC_GEMM_NT_RESID : OPTSTAGE_KC_GEMM_NT_STORE);
  KT(cls, 2.0 * M * N * K, gemm(st->sh, layout, epi, A, B, C, R, M, N, K, lda, ldb, ldc, st->cs));
  return OPTSTAGE_OK;
}
// the two projections with a fused epilogue (bf16 only)
optstage_status k_gemm_fused(optstage* st, int layout, int epi, const void* A, const void* B, void* C, int M, int N, int K,
                             int lda, int ldb, int ldc, const GemmExtra& ex) {
  KT(epi == EPI_ROPE ? OPTSTAGE_KC_GEMM_NT_QKV : OPTSTAGE_KC_GEMM_NT_GU, 2.0 * M * N * K,
     launch_gemm_bf16(layout, epi, A, B, C, nullptr, M, N, K, lda, ldb, ldc, st->cs, &ex));
  return OPTSTAGE_OK;
}
optstage_status k_gemm_grouped(optstage* st, int layout, int epi, int n, const GemmProblem* pr, int K) {
  double flops = 0;
  for (int i = 0; i < n; ++i) flops += 2.0 * pr[i].M * pr[i].N * K;
  KT(OPTSTAGE_KC_GEMM_TN_ACCUM, flops, launch_gemm_bf16_grouped(layout, epi, n, pr, K, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_norm_fwd(optstage* st, const void* x, const void* g, const void* b, void* out, float* stats) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_NORM_FWD, 2.0 * s.e * s.tokens * s.h, launch_norm_fwd(s.dtype, s.family, x, g, b, out, stats, s.tokens,
      s.h, st->desc.norm_eps, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_norm_bwd(optstage* st, const void* dn, const void* x, const float* stats, const void* g, const void* dres,
    void* dx, float* dg, float* db, bool store) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_NORM_BWD, 4.0 * s.e * s.tokens * s.h, launch_norm_bwd(s.dtype, s.family, dn, x, stats, g, dres, dx,
      (float*)(st->wsp() + st->ws.partial), dg, db, s.tokens, s.h, st->cs, store ? 1 : 0));
  return OPTSTAGE_OK;
}
optstage_status k_act_fwd(optstage* st, const void* gu, void* a) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_ACT_FWD, (s.family == OPTSTAGE_LLAMA ? 3.0 : 2.0) * s.e * s.tokens * s.f, launch_act_fwd(s.dtype, s.family,
      gu, a, s.tokens, s.f, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_act_bwd(optstage* st, const void* da, const void* gu, void* dgu) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_ACT_BWD, (s.family == OPTSTAGE_LLAMA ? 5.0 : 3.0) * s.e * s.tokens * s.f, launch_act_bwd(s.dtype, s.family,
      da, gu, dgu, s.tokens, s.f, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_rope(optstage* st, const void* src, void* dst, int backward) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_ROPE, 2.0 * s.e * s.tokens * (s.nq + s.nkv) * s.d, launch_rope(s.dtype, src, dst,
      (const float*)(st->wsp() + st->ws.rope), s.tokens, s.seq, s.nq, s.nkv, s.d, backward, 1, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_attn_fwd(optstage* st, const void* qkv, void* o, float* lse) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_ATTN_FWD, 2.0 * s.mb * s.seq * s.seq * s.nq * s.d, launch_attn_fwd(s.dtype, qkv, o, lse, s.seq, s.mb, s.nq, s.nkv, s.d, st->cs));
  return OPTSTAGE_OK;
}
optstage_status k_attn_bwd(optstage* st, const void* qkv, const void* o, const void* dout, const float* lse, void* dqkv) {
  const Shape& s = st->sh;
  KT(OPTSTAGE_KC_ATTN_BWD, 5.0 * s.mb * s.seq * s.seq * s.nq * s.d, launch_attn_bwd(s.dtype, qkv, o, dout, lse, dqkv,
      (float*)(st->wsp() + st->ws.attn), s.seq, s.mb, s.nq, s.nkv, s.d, st->cs));
  return OPTSTAGE_OK;
}

optstage_status check_weights(optstage* st, bool need_grads) {
  const bool gpt = st->sh.family == OPTSTAGE_GPT;
  for (int l = 0; l < st->sh.L; ++l)
    for (int k = 0; k < OPTSTAGE_N_WEIGHTS; ++k) {
      if (!gpt && (k == OPTSTAGE_W_B1 || k == OPTSTAGE_W_B2)) continue;
      if (!W(st, l, k)) return fail(OPTSTAGE_E_STATE, "layer %d weight %d not set", l, k);
      if (need_grads && !GW(st, l, k)) return fail(OPTSTAGE_E_STATE, "layer %d weight %d has no gradient accumulator", l, k);
    }
  return OPTSTAGE_OK;
}

optstage_status exec_forward(optstage* st, int j, int c, const OpBufs& ob) {
  const Shape& s = st->sh;
  hipStream_t cs = st->cs;
  const int T = s.tokens;
  auto P = [&](int l, int k) { return (void*)(st->arena() + ob.dev[(size_t)l * NK + k]); };
  const int l0 = c * s.Lc, l1 = l0 + s.Lc;
  const size_t io = (size_t)c * st->desc.n_microbatches + j;
  HIP_TRY(hipMemcpyAsync(P(l0, OPTSTAGE_K_X_IN), st->x_in[io], st->raw[OPTSTAGE_K_X_IN], hipMemcpyDeviceToDevice, cs));
  const int nstat = s.family == OPTSTAGE_LLAMA ? 1 : 2;
  const bool rc = st->lg.recompute;
  for (int l = l0; l < l1; ++l) {
    void* x = P(l, OPTSTAGE_K_X_IN);
    float* stats = (float*)P(l, OPTSTAGE_K_STATS);
    // not kept: the norm outputs and the MLP activation output live in B's transient buffers, idle during F
    void* n1 = rc ? (void*)(st->wsp() + st->ws.dn) : P(l, OPTSTAGE_K_N1);
    void* n2 = rc ? (void*)(st->wsp() + st->ws.dn) : P(l, OPTSTAGE_K_N2);
    void* a = rc ? (void*)(st->wsp() + st->ws.da) : P(l, OPTSTAGE_K_A);
    TRY(k_norm_fwd(st, x, W(st, l, OPTSTAGE_W_G1), W(st, l, OPTSTAGE_W_B1), n1, stats));
    int lay;
    const void* wq = fwd_operand(st, l, OPTSTAGE_W_QKV, &lay);
    if (s.fuse_rope) {
      GemmExtra ex;
      ex.table = (const float2*)(st->wsp() + st->ws.rope); ex.seq = s.seq; ex.rot_cols = (s.nq + s.nkv) * s.d;
      TRY(k_gemm_fused(st, lay, EPI_ROPE, n1, wq, P(l, OPTSTAGE_K_QKV), T, s.qkv_w, s.h, s.h, s.h, s.qkv_w, ex));
    } else {
      TRY(k_gemm(st, lay, EPI_STORE, n1, wq, P(l, OPTSTAGE_K_QKV), nullptr, T, s.qkv_w, s.h, s.h, s.h, s.qkv_w, OPTSTAGE_KC_GEMM_NT_QKV));
      if (s.family == OPTSTAGE_LLAMA)
        TRY(k_rope(st, P(l, OPTSTAGE_K_QKV), P(l, OPTSTAGE_K_QKV), 0));
    }
    TRY(k_attn_fwd(st, P(l, OPTSTAGE_K_QKV), P(l, OPTSTAGE_K_O), (float*)P(l, OPTSTAGE_K_LSE)));
    const void* wo = fwd_operand(st, l, OPTSTAGE_W_O, &lay);
    TRY(k_gemm(st, lay, EPI_RESID, P(l, OPTSTAGE_K_O), wo, P(l, OPTSTAGE_K_X_MID), x, T, s.h, s.nq * s.d, s.nq * s.d, s.nq * s.d, s.h));
    TRY(k_norm_fwd(st, P(l, OPTSTAGE_K_X_MID), W(st, l, OPTSTAGE_W_G2), W(st, l, OPTSTAGE_W_B2), n2, stats + (size_t)nstat * T));
    const void* wgu = fwd_operand(st, l, OPTSTAGE_W_GU, &lay);
    if (s.fuse_act) {                      // wgu is the paired slab copy: gate / up product and activation in one kernel
      GemmExtra ex;
      ex.a_out = a; ex.f = s.f;
      TRY(k_gemm_fused(st, GEMM_NT_SLAB, EPI_SWIGLU, n2, wgu, P(l, OPTSTAGE_K_GU), T, s.up_w, s.h, s.h, 64, s.up_w, ex));
    } else {
      TRY(k_gemm(st, lay, EPI_STORE, n2, wgu, P(l, OPTSTAGE_K_GU), nullptr, T, s.up_w, s.h, s.h, s.h, s.up_w, OPTSTAGE_KC_GEMM_NT_GU));
      TRY(k_act_fwd(st, P(l, OPTSTAGE_K_GU), a));
    }
    void* y = l + 1 < l1 ? P(l + 1, OPTSTAGE_K_X_IN) : st->y_out[io];
    const void* wd = fwd_operand(st, l, OPTSTAGE_W_D, &lay);
    TRY(k_gemm(st, lay, EPI_RESID, a, wd, y, P(l, OPTSTAGE_K_X_MID), T, s.h, s.f, s.f, s.f, s.h));
    // everything this layer keeps is final from here on: an offload of its activations may start while the layers
    // after it still run
    HIP_TRY(hipEventRecord(st->ev_fl[(size_t)j * s.L + l], cs));
  }
  return OPTSTAGE_OK;
}

optstage_status exec_backward_input(optstage* st, int j, int c, const OpBufs& ob) {
  const Shape& s = st->sh;
  hipStream_t cs = st->cs;
  const int T = s.tokens;
  auto P = [&](int l, int k) { return (void*)(st->arena() + ob.dev[(size_t)l * NK + k]); };
  char* ws = st->wsp();
  void *da = ws + st->ws.da, *dn = ws + st->ws.dn, *dout = ws + st->ws.dout, *dqkv = ws + st->ws.dqkv;
  const int nstat = s.family == OPTSTAGE_LLAMA ? 1 : 2;
  const bool rc = st->lg.recompute;
  const int l0 = c * s.Lc, l1 = l0 + s.Lc;
  const size_t io = (size_t)c * st->desc.n_microbatches + j;
  // B ops of a chunk run in micro-batch order, so micro-batch 0 is the iteration's first: in overwrite mode it
  // stores the norm parameters' gradients instead of adding to what the accumulators held
  const bool store = st->overwrite && j == 0;
  HIP_TRY(hipMemcpyAsync(P(l1 - 1, OPTSTAGE_K_DY), st->dy_out[io], st->raw[OPTSTAGE_K_DY], hipMemcpyDeviceToDevice, cs));
  for (int l = l1 - 1; l >= l0; --l) {
    void* dy = P(l, OPTSTAGE_K_DY);
    float* stats = (float*)P(l, OPTSTAGE_K_STATS);
    // da = dy W_d ; dgu = act'(gu) da (over gu) ; dn2 = dgu W_gu
    int lay;
    const void* wd = bwd_operand(st, l, OPTSTAGE_W_D, &lay);
    TRY(k_gemm(st, lay, EPI_STORE, dy, wd, da, nullptr, T, s.f, s.h, s.h, s.h, s.f));
    if (rc) TRY(k_act_fwd(st, P(l, OPTSTAGE_K_GU), P(l, OPTSTAGE_K_A)));   // W's operand, before gu is overwritten
    TRY(k_act_bwd(st, da, P(l, OPTSTAGE_K_GU), P(l, OPTSTAGE_K_GU)));
    const void* wgu = bwd_operand(st, l, OPTSTAGE_W_GU, &lay);
    TRY(k_gemm(st, lay, EPI_STORE, P(l, OPTSTAGE_K_GU), wgu, dn, nullptr, T, s.h, s.up_w, s.up_w, s.up_w, s.h));
    if (rc) TRY(k_norm_fwd(st, P(l, OPTSTAGE_K_X_MID), W(st, l, OPTSTAGE_W_G2), W(st, l, OPTSTAGE_W_B2), P(l,
        OPTSTAGE_K_N2), stats + (size_t)nstat * T));
    // dx_mid = dy + norm2'(dn2)
    TRY(k_norm_bwd(st, dn, P(l, OPTSTAGE_K_X_MID), stats + (size_t)nstat * T, W(st, l, OPTSTAGE_W_G2), dy, P(l,
        OPTSTAGE_K_DX_MID), GW(st, l, OPTSTAGE_W_G2), GW(st, l, OPTSTAGE_W_B2), store));
    // do = dx_mid W_o ; attention backward ; rotary backward into the qkv buffer
    const void* wo = bwd_operand(st, l, OPTSTAGE_W_O, &lay);
    TRY(k_gemm(st, lay, EPI_STORE, P(l, OPTSTAGE_K_DX_MID), wo, dout, nullptr, T, s.nq * s.d, s.h, s.h, s.h, s.nq * s.d));
    TRY(k_attn_bwd(st, P(l, OPTSTAGE_K_QKV), P(l, OPTSTAGE_K_O), dout, (const float*)P(l, OPTSTAGE_K_LSE), dqkv));
    if (s.family == OPTSTAGE_LLAMA)
      TRY(k_rope(st, dqkv, P(l, OPTSTAGE_K_QKV), 1));
    else
      HIP_TRY(hipMemcpyAsync(P(l, OPTSTAGE_K_QKV), dqkv, st->raw[OPTSTAGE_K_QKV], hipMemcpyDeviceToDevice, cs));
    // dn1 = dqkv W_qkv ; dx_in = dx_mid + norm1'(dn1)
    const void* wq = bwd_operand(st, l, OPTSTAGE_W_QKV, &lay);
    TRY(k_gemm(st, lay, EPI_STORE, P(l, OPTSTAGE_K_QKV), wq, dn, nullptr, T, s.h, s.qkv_w, s.qkv_w, s.qkv_w, s.h));
    if (rc) TRY(k_norm_fwd(st, P(l, OPTSTAGE_K_X_IN), W(st, l, OPTSTAGE_W_G1), W(st, l, OPTSTAGE_W_B1), P(l, OPTSTAGE_K_N1), stats));
    void* dx = l > l0 ? P(l - 1, OPTSTAGE_K_DY) : st->dx_in[io];
    TRY(k_norm_bwd(st, dn, P(l, OPTSTAGE_K_X_IN), stats, W(st, l, OPTSTAGE_W_G1), P(l, OPTSTAGE_K_DX_MID), dx, GW(st, l,
        OPTSTAGE_W_G1), GW(st, l, OPTSTAGE_W_B1), store));
  }
  return OPTSTAGE_OK;
}

optstage_status exec_backward_weight(optstage* st, int j, int c, const OpBufs& ob) {
  const Shape& s = st->sh;
  hipStream_t cs = st->cs;
  const int T = s.tokens;
  auto P = [&](int l, int k) { return (void*)(st->arena() + ob.dev[(size_t)l * NK + k]); };
  // dW += dY^T X for the four linears of every layer (fp32 accumulators).  None of these products depends on
  // another: bf16 stages hand them to one grouped launch per 16, so that only the last launch leaves a partly
  // filled round of workgroups; anything the grouped path does not take runs product by product.
  std::vector<GemmProblem> pr;
  for (int l = c * s.Lc; l < (c + 1) * s.Lc; ++l) {
    pr.push_back({P(l, OPTSTAGE_K_DY), P(l, OPTSTAGE_K_A), GW(st, l, OPTSTAGE_W_D), nullptr, s.h, s.f, s.h, s.f, s.f});
    pr.push_back({P(l, OPTSTAGE_K_GU), P(l, OPTSTAGE_K_N2), GW(st, l, OPTSTAGE_W_GU), nullptr, s.up_w, s.h, s.up_w, s.h, s.h});
    pr.push_back({P(l, OPTSTAGE_K_DX_MID), P(l, OPTSTAGE_K_O), GW(st, l, OPTSTAGE_W_O), nullptr, s.h, s.nq * s.d, s.h, s.nq * s.d, s.nq * s.d});
    pr.push_back({P(l, OPTSTAGE_K_QKV), P(l, OPTSTAGE_K_N1), GW(st, l, OPTSTAGE_W_QKV), nullptr, s.qkv_w, s.h, s.qkv_w, s.h, s.h});
  }
  // W ops of a chunk run in micro-batch order: in overwrite mode micro-batch 0 stores its products (no read of the
  // accumulators, and nobody has to clear them between iterations), the others add
  const int epi = st->overwrite && j == 0 ? EPI_STOREF : EPI_ACCUM;
  for (size_t i0 = 0; i0 < pr.size(); i0 += 16) {
    const int n = (int)std::min<size_t>(16, pr.size() - i0);
    const bool grouped = s.dtype == OPTSTAGE_BF16 && gemm_bf16_grouped_applies(GEMM_TN, n, &pr[i0], T);
    if (grouped) TRY(k_gemm_grouped(st, GEMM_TN, epi, n, &pr[i0], T));
    if (!grouped)
      for (int i = 0; i < n; ++i) {
        const GemmProblem& q = pr[i0 + i];
        TRY(k_gemm(st, GEMM_TN, epi, q.A, q.B, q.C, nullptr, q.M, q.N, T, q.lda, q.ldb, q.ldc));
      }
  }
  return OPTSTAGE_OK;
}

// enqueues the compute-stream wait for `n` events bracketed by a stall span
optstage_status timed_wait(optstage* st, const hipEvent_t* evs, int n, int trace) {
  TimedSpan sp;
  optstage_status rc = span_begin(st, SPAN_STALL, st->cs, &sp, trace);
  if (rc != OPTSTAGE_OK) return rc;
  for (int i = 0; i < n; ++i) HIP_TRY(hipStreamWaitEvent(st->cs, evs[i], 0));
  return span_end(st, st->cs, sp);
}

optstage_status exec_event(optstage* st, const optstage_event& ev, const OpBufs& ob, int ti) {
  const int j = ev.microbatch, L = st->sh.L, m = st->desc.n_microbatches;
  // F / B / W carry their chunk in the layer field; a transfer belongs to the chunk that holds its layer
  const int c = ev.op <= OPTSTAGE_W ? (int)ev.layer : (int)ev.layer / st->sh.Lc;
  hipEvent_t ev_f = st->ev_f[(size_t)c * m + j];
  TimedSpan sp;
  optstage_status rc;
  switch (ev.op) {
    case OPTSTAGE_F:
      if ((rc = span_begin(st, ev.op, st->cs, &sp, ti)) != OPTSTAGE_OK) return rc;
      if ((rc = exec_forward(st, j, c, ob)) != OPTSTAGE_OK) return rc;
      if ((rc = span_end(st, st->cs, sp)) != OPTSTAGE_OK) return rc;
      HIP_TRY(hipEventRecord(ev_f, st->cs));
      break;
    case OPTSTAGE_B:
      // every reload of this micro-batch must have completed (the reload ends before its consumer starts); an
      // event that was not recorded in this iteration holds an older, completed record
      if (st->reloaded[(size_t)c * m + j]) {
        if ((rc = timed_wait(st, &st->ev_r[(size_t)j * L + c * st->sh.Lc], st->sh.Lc, ti)) != OPTSTAGE_OK) return rc;
      }
      if ((rc = span_begin(st, ev.op, st->cs, &sp, ti)) != OPTSTAGE_OK) return rc;
      if ((rc = exec_backward_input(st, j, c, ob)) != OPTSTAGE_OK) return rc;
      if ((rc = span_end(st, st->cs, sp)) != OPTSTAGE_OK) return rc;
      break;
    case OPTSTAGE_W:
      if ((rc = span_begin(st, ev.op, st->cs, &sp, ti)) != OPTSTAGE_OK) return rc;
      if ((rc = exec_backward_weight(st, j, c, ob)) != OPTSTAGE_OK) return rc;
      if ((rc = span_end(st, st->cs, sp)) != OPTSTAGE_OK) return rc;
      break;
    case OPTSTAGE_O: {
      // the offload starts once the layer that produced the data has ended (the F it belongs to may still be running
      // its later layers; the list has the O after that F, so the layer's event has been recorded)
      (void)ev_f;
      HIP_TRY(hipStreamWaitEvent(st->xs, st->ev_fl[(size_t)j * L + ev.layer], 0));
      // a pinned slot released by a reload listed earlier may be handed to this offload: with a reload stream
      // of its own that reload must have drained first (on a shared channel stream order already says so)
      if (st->rs != st->xs && st->last_r) HIP_TRY(hipStreamWaitEvent(st->xs, st->last_r, 0));
      if ((rc = span_begin(st, ev.op, st->xs, &sp, ti)) != OPTSTAGE_OK) return rc;
      for (int k = 0; k < NFK; ++k)
        if (ev.kind_mask & (1u << k)) {
          size_t i = (size_t)ev.layer * NK + k;
          HIP_TRY(hipMemcpyAsync((char*)st->desc.host_pool + ob.host[i], st->arena() + ob.dev[i], st->raw[k], hipMemcpyDeviceToHost, st->xs));
          st->stats.bytes_offloaded += st->raw[k];
        }
      if ((rc = span_end(st, st->xs, sp)) != OPTSTAGE_OK) return rc;
      HIP_TRY(hipEventRecord(st->ev_o[(size_t)j * L + ev.layer], st->xs));
      break;
    }
    case OPTSTAGE_OWAIT:
      // compute ops listed from here on may reuse the freed bytes: they start after the offload ended
      if ((rc = timed_wait(st, &st->ev_o[(size_t)j * L + ev.layer], 1, ti)) != OPTSTAGE_OK) return rc;
      break;
    case OPTSTAGE_R: {
      // the reload starts after the compute ops listed before it have ended
      hipEvent_t pos = st->ev_pos[(size_t)j * L + ev.layer];
      HIP_TRY(hipEventRecord(pos, st->cs));
      HIP_TRY(hipStreamWaitEvent(st->rs, pos, 0));
      // ... and after the offload that filled the host slot (implied by stream order on a shared channel)
      if (st->rs != st->xs) HIP_TRY(hipStreamWaitEvent(st->rs, st->ev_o[(size_t)j * L + ev.layer], 0));
      if ((rc = span_begin(st, ev.op, st->rs, &sp, ti)) != OPTSTAGE_OK) return rc;
      for (int k = 0; k < NFK; ++k)
        if (ev.kind_mask & (1u << k)) {
          size_t i = (size_t)ev.layer * NK + k;
          HIP_TRY(hipMemcpyAsync(st->arena() + ob.dev[i], (char*)st->desc.host_pool + ob.host[i], st->raw[k], hipMemcpyHostToDevice, st->rs));
          st->stats.bytes_reloaded += st->raw[k];
        }
      if ((rc = span_end(st, st->rs, sp)) != OPTSTAGE_OK) return rc;
      HIP_TRY(hipEventRecord(st->ev_r[(size_t)j * L + ev.layer], st->rs));
      st->last_r = st->ev_r[(size_t)j * L + ev.layer];
      st->reloaded[(size_t)c * m + j] = 1;
      break;
    }
  }
  st->stats.n_ops[ev.op]++;
  return OPTSTAGE_OK;
}

optstage_status precheck(optstage* st, const optstage_event* events, size_t n) {
  bool needs_host = false;
  for (size_t i = 0; i < n; ++i) {
    const optstage_event& ev = events[i];
    if (ev.op > OPTSTAGE_R) return fail(OPTSTAGE_E_ARG, "event %zu: unknown op %u", i, ev.op);
    if (ev.microbatch >= st->desc.n_microbatches) return fail(OPTSTAGE_E_ARG, "event %zu: micro-batch out of range", i);
    const int j = ev.microbatch;
    if (ev.op <= OPTSTAGE_W && ev.layer >= (uint32_t)st->sh.chunks) return fail(OPTSTAGE_E_ARG, "event %zu: chunk %u out of range", i, ev.layer);
    if (ev.op > OPTSTAGE_W && ev.layer >= (uint32_t)st->sh.L) return fail(OPTSTAGE_E_ARG, "event %zu: layer %u out of range", i, ev.layer);
    const size_t io = ev.op <= OPTSTAGE_W ? (size_t)ev.layer * st->desc.n_microbatches + j : 0;
    if (ev.op == OPTSTAGE_F && (!st->x_in[io] || !st->y_out[io])) return fail(OPTSTAGE_E_STATE,
        "event %zu: x_in / y_out of micro-batch %d not bound", i, j);
    if (ev.op == OPTSTAGE_B && (!st->dy_out[io] || !st->dx_in[io])) return fail(OPTSTAGE_E_STATE,
        "event %zu: dy_out / dx_in of micro-batch %d not bound", i, j);
    if (ev.op == OPTSTAGE_O) needs_host = true;
  }
  if (needs_host && !st->desc.host_pool) return fail(OPTSTAGE_E_HOSTPOOL, "offload requested but no pinned host pool was given");
  bool any_bw = false;
  for (size_t i = 0; i < n; ++i) any_bw |= events[i].op == OPTSTAGE_B || events[i].op == OPTSTAGE_W;
  return check_weights(st, any_bw);
}

optstage_status run_list(optstage* st, const optstage_event* events, size_t n) {
  if (!st || (!events && n)) return fail(OPTSTAGE_E_ARG, "null argument");
  if (st->failed) return fail(OPTSTAGE_E_STATE, "an earlier call failed while enqueueing: call optstage_synchronize and optstage_reset");
  optstage_status rc = precheck(st, events, n);
  if (rc != OPTSTAGE_OK) return rc;
  {
    Logical trial = st->lg;   // validate on a copy: a failing list changes nothing
    for (size_t i = 0; i < n; ++i)
      if ((rc = apply_event(trial, events[i], nullptr)) != OPTSTAGE_OK) {
        char tmp[400];
        snprintf(tmp, sizeof tmp, "%s", g_err);
        return fail(rc, "event %zu: %s", i, tmp);
      }
  }
  if (n && !st->origin_set) {
    HIP_TRY(hipEventRecord(st->origin, st->cs));
    st->origin_set = true;
  }
  OpBufs ob;
  for (size_t i = 0; i < n; ++i) {
    if ((rc = apply_event(st->lg, events[i], &ob)) != OPTSTAGE_OK) return rc;   // cannot fail: same steps as the trial
    if (events[i].op == OPTSTAGE_F) st->in_flight++;
    if (events[i].op == OPTSTAGE_W) st->in_flight--;
    st->sum_live += (double)st->lg.live;
    if (st->in_flight && st->lg.live < st->min_live) st->min_live = st->lg.live;
    optstage_trace_entry te;
    memset(&te, 0, sizeof te);
    te.op = events[i].op; te.microbatch = events[i].microbatch; te.layer = events[i].layer; te.kind_mask = events[i].kind_mask;
    te.live_bytes = st->lg.live;
    te.start_ms = te.end_ms = -1.0;
    st->trace.push_back(te);
    if ((rc = exec_event(st, events[i], ob, (int)st->trace.size() - 1)) != OPTSTAGE_OK) {
      // the accounting is ahead of what was enqueued and an op graph may be half launched: nothing more runs on
      // this handle until optstage_reset
      st->failed = true;
      return rc;
    }
  }
  return OPTSTAGE_OK;
}

// empty accounting state for one iteration; lg.bytes is left alone
void init_logical(Logical& lg, const Shape& s, const optstage_desc& d, uint64_t arena_cap, uint64_t host_cap) {
  lg.L = s.L;
  lg.chunks = s.chunks;
  lg.Lc = s.Lc;
  lg.m = d.n_microbatches;
  lg.budget = d.hbm_budget_bytes;
  lg.recompute = d.recompute != 0;
  lg.live = lg.peak = 0;
  lg.next_f.assign(s.chunks, 0);
  lg.next_b.assign(s.chunks, 0);
  lg.next_w.assign(s.chunks, 0);
  lg.mbs.assign((size_t)lg.m * s.chunks, MbState());
  lg.bufs.assign((size_t)lg.m * lg.L * NK, BufRec());
  lg.arena.reset(arena_cap);
  lg.host.reset(host_cap);
}

void reset_logical(optstage* st) {
  init_logical(st->lg, st->sh, st->desc, st->desc.arena_bytes / ALIGN * ALIGN,
               st->desc.host_pool ? st->desc.host_pool_bytes / ALIGN * ALIGN : 0);
}

}  // namespace

extern "C" {

const char* optstage_last_error(void) { return g_err; }

optstage_status optstage_query_sizes(const optstage_desc* desc, uint64_t* min_workspace, uint64_t* act_bytes_per_mb,
                                     uint64_t* bytes_per_kind) {
  Shape s;
  optstage_status rc = shape_from_desc(desc, &s);
  if (rc != OPTSTAGE_OK) return rc;
  uint64_t raw[NK];
  kind_raw_bytes(s, raw);
  uint64_t per_layer = 0;
  for (int k = 0; k < NK; ++k) {
    if (bytes_per_kind) bytes_per_kind[k] = round_up(raw[k]);
    if (k < NFK && !(desc->recompute && recomputable(k))) per_layer += round_up(raw[k]);
  }
  if (act_bytes_per_mb) *act_bytes_per_mb = per_layer * s.L;
  if (min_workspace) *min_workspace = workspace_layout(s).total;
  return OPTSTAGE_OK;
}

optstage_status optstage_create(const optstage_desc* desc, optstage_t** out) {
  if (!out) return fail(OPTSTAGE_E_ARG, "out is null");
  *out = nullptr;
  Shape s;
  optstage_status rc = shape_from_desc(desc, &s);
  if (rc != OPTSTAGE_OK) return rc;
  if (!desc->arena || !desc->workspace) return fail(OPTSTAGE_E_ARG, "arena and workspace must be given");
  if (((uintptr_t)desc->arena | (uintptr_t)desc->workspace | (uintptr_t)desc->host_pool) & (ALIGN - 1))
    return fail(OPTSTAGE_E_ARG, "arena, workspace and host_pool must be 256-byte aligned");
  WorkspaceLayout ws = workspace_layout(s);
  if (desc->workspace_bytes < ws.total)
    return fail(OPTSTAGE_E_ARG, "workspace_bytes %llu < required %llu", (unsigned long long)desc->workspace_bytes, (unsigned long long)ws.total);
  optstage* st = new (std::nothrow) optstage();
  if (!st) return fail(OPTSTAGE_E_ARG, "out of host memory");
  st->desc = *desc;
  st->sh = s;
  st->ws = ws;
  kind_raw_bytes(s, st->raw);
  for (int k = 0; k < NK; ++k) {
    st->lg.bytes[k] = round_up(st->raw[k]);
    if (st->raw[k] % 8) { delete st; return fail(OPTSTAGE_E_ARG, "activation kind %d is not a multiple of 8 bytes", k); }
  }
  st->cs = (hipStream_t)desc->compute_stream;
  st->xs = (hipStream_t)desc->copy_stream;
  st->rs = desc->reload_stream ? (hipStream_t)desc->reload_stream : st->xs;
  const size_t m = desc->n_microbatches, L = s.L;
  st->w.assign(L * OPTSTAGE_N_WEIGHTS, nullptr);
  st->gw.assign(L * OPTSTAGE_N_WEIGHTS, nullptr);
  const size_t nio = m * s.chunks;   // [chunk][mb]
  st->x_in.assign(nio, nullptr); st->dy_out.assign(nio, nullptr); st->y_out.assign(nio, nullptr); st->dx_in.assign(nio, nullptr);
  memset(&st->stats, 0, sizeof st->stats);
  reset_logical(st);
  auto mk = [&](std::vector<hipEvent_t>& v, size_t n) -> bool {
    v.assign(n, nullptr);
    for (size_t i = 0; i < n; ++i)
      if (hipEventCreateWithFlags(&v[i], hipEventDisableTiming) != hipSuccess) return false;
    return true;
  };
  st->reloaded.assign(nio, 0);
  if (hipError_t e = hipEventCreate(&st->origin); e != hipSuccess) {
    st->origin = nullptr;
    optstage_destroy(st);
    return fail(OPTSTAGE_E_HIP, "hipEventCreate: %s", hipGetErrorString(e));
  }
  if (!mk(st->ev_f, nio) || !mk(st->ev_o, m * L) || !mk(st->ev_r, m * L) || !mk(st->ev_pos, m * L) || !mk(st->ev_fl, m * L)) {
    optstage_destroy(st);
    return fail(OPTSTAGE_E_HIP, "hipEventCreateWithFlags failed");
  }
  // an event that was never recorded counts as complete, so B may wait on every ev_r unconditionally
  if (s.family == OPTSTAGE_LLAMA) {
    hipError_t e = launch_rope_table((float*)(st->wsp() + ws.rope), s.seq, s.d, desc->rope_base, st->cs);
    if (e != hipSuccess) { optstage_destroy(st); return fail(OPTSTAGE_E_HIP, "rope table: %s", hipGetErrorString(e)); }
  }
  *out = st;
  return OPTSTAGE_OK;
}

void optstage_destroy(optstage_t* st) {
  if (!st) return;
  for (auto* v : {&st->ev_f, &st->ev_o, &st->ev_r, &st->ev_pos, &st->ev_fl, &st->tpool})
    for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
  if (st->origin) (void)hipEventDestroy(st->origin);
  delete st;
}

optstage_status optstage_set_weight(optstage_t* st, uint32_t layer, uint32_t which, const void* weight_dev, float* grad) {
  if (!st || !weight_dev) return fail(OPTSTAGE_E_ARG, "null argument");
  if (layer >= (uint32_t)st->sh.L || which >= OPTSTAGE_N_WEIGHTS) return fail(OPTSTAGE_E_ARG, "layer or weight id out of range");
  if (st->sh.family == OPTSTAGE_LLAMA && (which == OPTSTAGE_W_B1 || which == OPTSTAGE_W_B2)) return fail(OPTSTAGE_E_ARG,
      "this family has no norm bias");
  if (((uintptr_t)weight_dev | (uintptr_t)grad) & 15) return fail(OPTSTAGE_E_ARG, "weights and gradients must be 16-byte aligned");
  st->w[(size_t)layer * OPTSTAGE_N_WEIGHTS + which] = weight_dev;
  st->gw[(size_t)layer * OPTSTAGE_N_WEIGHTS + which] = grad;
  const Shape& s = st->sh;
  int rows = 0, cols = 0;
  if (!weight_dims(s, which, &rows, &cols)) return OPTSTAGE_OK;
  bool sf, sb;
  slab_modes(s, which, &sf, &sb);
  if (sb) HIP_TRY(launch_slabs(weight_dev, (void*)WT(st, layer, which), cols, rows, 1, st->cs));
  else HIP_TRY(launch_transpose(s.dtype, weight_dev, (void*)WT(st, layer, which), rows, cols, st->cs));
  // the forward copy of the gate / up weight is in paired slabs when the activation runs in that product's epilogue
  if (sf) HIP_TRY(launch_slabs(weight_dev, (void*)WF(st, layer, which), rows, cols, which == OPTSTAGE_W_GU && s.fuse_act ? 2 : 0, st->cs));
  return OPTSTAGE_OK;
}

optstage_status optstage_bind_io_chunk(optstage_t* st, uint32_t chunk, uint32_t mb, const void* x_in, const void* dy_out,
                                       void* y_out, void* dx_in) {
  if (!st) return fail(OPTSTAGE_E_ARG, "null handle");
  if (chunk >= (uint32_t)st->sh.chunks) return fail(OPTSTAGE_E_ARG, "chunk out of range");
  if (mb >= st->desc.n_microbatches) return fail(OPTSTAGE_E_ARG, "micro-batch out of range");
  if (((uintptr_t)x_in | (uintptr_t)dy_out | (uintptr_t)y_out | (uintptr_t)dx_in) & 15) return fail(OPTSTAGE_E_ARG,
      "io tensors must be 16-byte aligned");
  const size_t io = (size_t)chunk * st->desc.n_microbatches + mb;
  st->x_in[io] = x_in; st->dy_out[io] = dy_out; st->y_out[io] = y_out; st->dx_in[io] = dx_in;
  return OPTSTAGE_OK;
}

optstage_status optstage_bind_io(optstage_t* st, uint32_t mb, const void* x_in, const void* dy_out, void* y_out, void* dx_in) {
  return optstage_bind_io_chunk(st, 0, mb, x_in, dy_out, y_out, dx_in);
}

optstage_status optstage_validate(const optstage_t* st, const optstage_event* events, size_t n, size_t* first_bad) {
  if (!st || (!events && n)) return fail(OPTSTAGE_E_ARG, "null argument");
  Logical lg;
  memcpy(lg.bytes, st->lg.bytes, sizeof lg.bytes);
  init_logical(lg, st->sh, st->desc, st->desc.arena_bytes / ALIGN * ALIGN,
               st->desc.host_pool ? st->desc.host_pool_bytes / ALIGN * ALIGN : 0);
  for (size_t i = 0; i < n; ++i) {
    optstage_status rc = apply_event(lg, events[i], nullptr);
    if (rc != OPTSTAGE_OK) {
      if (first_bad) *first_bad = i;
      return rc;
    }
  }
  optstage_status rc = check_complete(lg);
  if (rc == OPTSTAGE_OK)
    for (auto& b : lg.bufs)
      if (b.state == B_OFFLOADING || b.state == B_HOST) { rc = fail(OPTSTAGE_E_ORDER, "an offloaded activation is never reloaded"); break; }
  if (rc != OPTSTAGE_OK && first_bad) *first_bad = n;
  return rc;
}

optstage_status optstage_plan(const optstage_desc* desc, const optstage_event* events, size_t n, size_t* first_bad,
                              uint64_t* peak_bytes, uint64_t* live_after) {
  Shape s;
  optstage_status rc = shape_from_desc(desc, &s);
  if (rc != OPTSTAGE_OK) return rc;
  if (!events && n) return fail(OPTSTAGE_E_ARG, "events is null");
  uint64_t raw[NK];
  kind_raw_bytes(s, raw);
  Logical lg;
  for (int k = 0; k < NK; ++k) lg.bytes[k] = round_up(raw[k]);
  // logical accounting only: unbounded placement space
  init_logical(lg, s, *desc, UINT64_MAX / 2 / ALIGN * ALIGN, UINT64_MAX / 2 / ALIGN * ALIGN);
  if (peak_bytes) *peak_bytes = 0;
  for (size_t i = 0; i < n; ++i) {
    rc = apply_event(lg, events[i], nullptr);
    if (peak_bytes) *peak_bytes = lg.peak;
    if (rc != OPTSTAGE_OK) {
      if (first_bad) *first_bad = i;
      return rc;
    }
    if (live_after) live_after[i] = lg.live;
  }
  rc = check_complete(lg);
  if (rc == OPTSTAGE_OK)
    for (auto& b : lg.bufs)
      if (b.state == B_OFFLOADING || b.state == B_HOST) { rc = fail(OPTSTAGE_E_ORDER, "an offloaded activation is never reloaded"); break; }
  if (rc != OPTSTAGE_OK && first_bad) *first_bad = n;
  return rc;
}

optstage_status optstage_run(optstage_t* st, const optstage_event* events, size_t n) { return run_list(st, events, n); }

static optstage_status one(optstage_t* st, uint32_t op, uint32_t mb, uint32_t layer, uint32_t mask) {
  optstage_event ev = {op, mb, layer, mask};
  return run_list(st, &ev, 1);
}
optstage_status optstage_forward(optstage_t* st, uint32_t mb) { return one(st, OPTSTAGE_F, mb, 0, 0); }
optstage_status optstage_backward_input(optstage_t* st, uint32_t mb) { return one(st, OPTSTAGE_B, mb, 0, 0); }
optstage_status optstage_backward_weight(optstage_t* st, uint32_t mb) { return one(st, OPTSTAGE_W, mb, 0, 0); }
optstage_status optstage_offload(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t mask) { return one(st, OPTSTAGE_O, mb, layer, mask); }
optstage_status optstage_offload_wait(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t mask) { return one(st, OPTSTAGE_OWAIT, mb, layer, mask); }
optstage_status optstage_reload(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t mask) { return one(st, OPTSTAGE_R, mb, layer, mask); }

optstage_status optstage_synchronize(optstage_t* st) {
  if (!st) return fail(OPTSTAGE_E_ARG, "null handle");
  HIP_TRY(hipStreamSynchronize(st->cs));
  HIP_TRY(hipStreamSynchronize(st->xs));
  if (st->rs != st->xs) HIP_TRY(hipStreamSynchronize(st->rs));
  for (const TimedSpan& sp : st->spans) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
    if (sp.op == SPAN_STALL) {
      const bool reload = sp.trace >= 0 && st->trace[sp.trace].op == OPTSTAGE_B;
      st->stats.stall_ms[reload ? 1 : 0] += ms;
      if (sp.trace >= 0) st->trace[sp.trace].stall_ms += ms;
    } else if (sp.op >= 0) {
      st->stats.ms_ops[sp.op] += ms;
      if (sp.trace >= 0 && st->origin_set) {
        float t0 = 0.f;
        HIP_TRY(hipEventElapsedTime(&t0, st->origin, sp.a));
        st->trace[sp.trace].start_ms = t0;
        st->trace[sp.trace].end_ms = t0 + ms;
      }
    } else {
      st->stats.kernel_ms[-sp.op - 1] += ms;
    }
  }
  st->spans.clear();
  st->tnext = 0;
  return OPTSTAGE_OK;
}

optstage_status optstage_reset(optstage_t* st) {
  if (!st) return fail(OPTSTAGE_E_ARG, "null handle");
  if (!st->spans.empty()) return fail(OPTSTAGE_E_STATE, "reset with work in flight: call optstage_synchronize first");
  reset_logical(st);
  memset(&st->stats, 0, sizeof st->stats);
  st->last_r = nullptr;
  st->failed = false;
  st->origin_set = false;
  st->trace.clear();
  std::fill(st->reloaded.begin(), st->reloaded.end(), 0);
  st->in_flight = 0;
  st->min_live = UINT64_MAX;
  st->sum_live = 0.0;
  return OPTSTAGE_OK;
}

optstage_status optstage_set_kernel_timing(optstage_t* st, uint32_t on) {
  if (!st) return fail(OPTSTAGE_E_ARG, "null handle");
  st->ktiming = on != 0;
  return OPTSTAGE_OK;
}

optstage_status optstage_get_stats(optstage_t* st, optstage_stats* out) {
  if (!st || !out) return fail(OPTSTAGE_E_ARG, "null argument");
  *out = st->stats;
  out->live_bytes = st->lg.live;
  out->peak_bytes = st->lg.peak;
  out->arena_high_water = st->lg.arena.high_water();
  out->n_trace = st->trace.size();
  out->min_live_bytes = st->min_live == UINT64_MAX ? 0 : st->min_live;
  out->avg_live_bytes = st->trace.empty() ? 0.0 : st->sum_live / (double)st->trace.size();
  return OPTSTAGE_OK;
}

optstage_status optstage_get_trace(optstage_t* st, optstage_trace_entry* out, size_t capacity, size_t* n_total) {
  if (!st || (!out && capacity)) return fail(OPTSTAGE_E_ARG, "null argument");
  if (n_total) *n_total = st->trace.size();
  const size_t n = std::min(capacity, st->trace.size());
  if (n) memcpy(out, st->trace.data(), n * sizeof(optstage_trace_entry));
  return OPTSTAGE_OK;
}

optstage_status optstage_set_grad_overwrite(optstage_t* st, uint32_t on) {
  if (!st) return fail(OPTSTAGE_E_ARG, "null handle");
  st->overwrite = on != 0;
  return OPTSTAGE_OK;
}

optstage_status optstage_debug_checksum(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind, uint32_t where, uint64_t* out) {
  if (!st || !out) return fail(OPTSTAGE_E_ARG, "null argument");
  if (mb >= st->desc.n_microbatches || layer >= (uint32_t)st->sh.L || kind >= NK || where > 1) return fail(OPTSTAGE_E_ARG, "index out of range");
  const BufRec& b = st->lg.buf(mb, layer, kind);
  HIP_TRY(hipStreamSynchronize(st->cs));
  HIP_TRY(hipStreamSynchronize(st->xs));
  if (st->rs != st->xs) HIP_TRY(hipStreamSynchronize(st->rs));
  if (where == 0) {
    if (b.state != B_DEV && b.state != B_OFFLOADING && b.state != B_RELOADED) return fail(OPTSTAGE_E_STATE, "buffer has no device copy");
    uint64_t* dev = (uint64_t*)(st->wsp() + st->ws.csum);
    HIP_TRY(launch_checksum(st->arena() + b.dev_off, st->raw[kind], dev, st->cs));
    HIP_TRY(hipMemcpyAsync(out, dev, 16, hipMemcpyDeviceToHost, st->cs));
    HIP_TRY(hipStreamSynchronize(st->cs));
  } else {
    if (b.state != B_OFFLOADING && b.state != B_HOST) return fail(OPTSTAGE_E_STATE, "buffer has no host copy");
    const uint64_t* p = (const uint64_t*)((char*)st->desc.host_pool + b.host_off);
    uint64_t s = 0, x = 0;
    for (uint64_t i = 0; i < st->raw[kind] / 8; ++i) { s += p[i]; x ^= p[i]; }
    out[0] = s; out[1] = x;
  }
  return OPTSTAGE_OK;
}

optstage_status optstage_debug_read(optstage_t* st, uint32_t mb, uint32_t layer, uint32_t kind, void* dst, uint64_t dst_bytes) {
  if (!st || !dst) return fail(OPTSTAGE_E_ARG, "null argument");
  if (mb >= st->desc.n_microbatches || layer >= (uint32_t)st->sh.L || kind >= NK) return fail(OPTSTAGE_E_ARG, "index out of range");
  if (dst_bytes < st->raw[kind]) return fail(OPTSTAGE_E_ARG, "dst too small: need %llu bytes", (unsigned long long)st->raw[kind]);
  const BufRec& b = st->lg.buf(mb, layer, kind);
  if (b.state != B_DEV && b.state != B_OFFLOADING && b.state != B_RELOADED) return fail(OPTSTAGE_E_STATE, "buffer has no device copy");
  HIP_TRY(hipStreamSynchronize(st->xs));
  if (st->rs != st->xs) HIP_TRY(hipStreamSynchronize(st->rs));      // a reload into this buffer may be in flight there
  HIP_TRY(hipMemcpyAsync(dst, st->arena() + b.dev_off, st->raw[kind], hipMemcpyDeviceToHost, st->cs));
  HIP_TRY(hipStreamSynchronize(st->cs));
  return OPTSTAGE_OK;
}

}  // extern "C"
