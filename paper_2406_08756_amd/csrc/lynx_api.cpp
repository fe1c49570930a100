// Host runtime behind the C ABI: configuration checks, the 13-operator graph,
// residency bookkeeping over the workspace allocator, and the operator /
// gradient sequences that enqueue the HIP kernels.
//
// Every state-changing call is executed twice: first as a rehearsal on a copy
// of the bookkeeping with launching disabled (so dependency and out-of-memory
// errors surface before anything is enqueued or changed), then for real.  The
// allocator is deterministic, so both passes see the same offsets.
#include <hip/hip_runtime.h>
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/lynx.h"
#include "arena.h"
#include "kernels.h"
#include "static_workspace.h"

namespace {

using lynx::Arena;
using lynx::GemmDesc;

constexpr int kNumAct = LYNX_NUM_ACTIVATIONS;
constexpr int kNumOps = 13;

// activations each operator reads (-1 terminated)
constexpr int kParents[kNumOps + 1][3] = {
    {-1, -1, -1}, {0, -1, -1}, {1, -1, -1}, {2, -1, -1}, {3, -1, -1}, {4, -1, -1}, {5, 2, -1},
    {6, -1, -1},  {0, 7, -1},  {8, -1, -1}, {9, -1, -1}, {10, -1, -1}, {11, -1, -1}, {8, 12, -1}};
// the last forward operator that reads each activation (0 = none)
constexpr int kLastForwardUse[kNumAct] = {8, 2, 6, 4, 5, 6, 7, 8, 13, 10, 11, 12, 13, 0};
// activations the backward pass reads
constexpr uint32_t kBackwardNeeds = (1u << 0) | (1u << 1) | (1u << 2) | (1u << 4) | (1u << 5) |
                                    (1u << 6) | (1u << 8) | (1u << 9) | (1u << 10) | (1u << 11);
constexpr uint32_t kCallerOwned = (1u << 0) | (1u << 13);

struct Dims {
  int dtype, e;
  int b, s, a, d, h, p, f, T;
  size_t ss;  // b * a * s * s
};

bool make_dims(const lynx_layer_config* c, Dims* o) {
  if (c == nullptr) return false;
  if (c->dtype != LYNX_F32 && c->dtype != LYNX_BF16) return false;
  if (c->hidden <= 0 || c->local_heads <= 0 || c->head_dim <= 0 || c->local_ffn <= 0 ||
      c->seq <= 0 || c->micro_batch <= 0)
    return false;
  if (c->hidden % 8 || c->head_dim % 8 || c->local_ffn % 8 || c->seq % 8) return false;
  if (c->hidden > 8192 || c->seq > 8192) return false;
  if (!(c->dropout_p >= 0.0f && c->dropout_p < 1.0f)) return false;
  if (!(c->ln_eps >= 0.0f)) return false;
  if (c->tp_size <= 0 || c->tp_rank < 0 || c->tp_rank >= c->tp_size) return false;
  if (c->layer_id >= (1u << 30) || c->causal != 1 || (c->flags & ~LYNX_FLAG_FUSED_ATTENTION)) return false;
  const long long T = static_cast<long long>(c->micro_batch) * c->seq;
  if (T > (1ll << 24)) return false;
  o->dtype = c->dtype;
  o->e = c->dtype == LYNX_BF16 ? 2 : 4;
  o->b = c->micro_batch; o->s = c->seq; o->a = c->local_heads; o->d = c->head_dim;
  o->h = c->hidden; o->p = c->local_heads * c->head_dim; o->f = c->local_ffn;
  o->T = static_cast<int>(T);
  o->ss = static_cast<size_t>(o->b) * o->a * o->s * o->s;
  return true;
}

size_t act_bytes(const Dims& D, int i) {
  const size_t th = static_cast<size_t>(D.T) * D.h * D.e;
  const size_t stats = 2 * static_cast<size_t>(D.T) * sizeof(float);
  switch (i) {
    case 0: case 7: case 8: case 12: case 13: return th;
    case 1: case 9: return th + stats;
    case 2: return static_cast<size_t>(D.T) * 3 * D.p * D.e;
    case 3: case 4: case 5: return D.ss * D.e;
    // C carries the attention row statistics (maximum, 1 / sum: two fp32 per row and head)
    // that the kernels which never store S, P, Pd leave for their backward
    case 6: return static_cast<size_t>(D.T) * D.p * D.e + static_cast<size_t>(D.b) * D.a * D.s * 2 * sizeof(float);
    case 10: case 11: return static_cast<size_t>(D.T) * D.f * D.e;
    default: return 0;
  }
}

// Residency bookkeeping: copyable, so calls can be rehearsed.
struct Book {
  Arena arena;
  bool live[kNumAct] = {};
  size_t off[kNumAct] = {};
  uint32_t retain = 0;
  int state = 0;  // 0 idle, 1 forward done / backward pending
  // the policy keeps none of S, P, Pd and the shape is one the fused attention kernels take:
  // operators 3-5 never run, operator 6 reads QKV alone
  bool fused_attn = false;
};

}  // namespace

struct lynx_layer_s {
  lynx_layer_config cfg;
  Dims D;
  char* base = nullptr;
  Book book;
  bool dry = false;
  bool have_params = false;
  lynx_params params{};
  const void* x = nullptr;
  void* out = nullptr;
  uint64_t step = 0;
  // optional per-kernel timing (the paper's Model Profiler collects operator
  // execution times C_i): one begin/end event pair per slot
  bool profiling = false;
  hipEvent_t ev_begin[LYNX_PROFILE_SLOTS] = {};
  hipEvent_t ev_end[LYNX_PROFILE_SLOTS] = {};
  bool ev_recorded[LYNX_PROFILE_SLOTS] = {};
  // parity aid: where backward copies the gradient with respect to activation A_i (null: nowhere)
  void* grad_tap[LYNX_NUM_ACTIVATIONS] = {};
  int static_device = -1;  // >= 0: the workspace is that device's built-in block
};

namespace {

struct Ctx {  // one pass (rehearsal or real) of a call
  lynx_layer_s* L;
  Book* bk;
  bool launch;
  hipStream_t st;
  hipError_t hip = hipSuccess;
};

#define LYNX_TRY(expr)                      \
  do {                                      \
    const lynx_status _s = (expr);          \
    if (_s != LYNX_OK) return _s;           \
  } while (0)

#define LYNX_LAUNCH(cx, slot, expr)                                            \
  do {                                                                         \
    if ((cx).launch) {                                                         \
      lynx_layer_s* _L = (cx).L;                                               \
      if (_L->profiling) (void)hipEventRecord(_L->ev_begin[slot], (cx).st);    \
      const hipError_t _e = (expr);                                            \
      if (_e != hipSuccess) { (cx).hip = _e; return LYNX_ERR_HIP; }            \
      if (_L->profiling) {                                                     \
        (void)hipEventRecord(_L->ev_end[slot], (cx).st);                       \
        _L->ev_recorded[slot] = true;                                          \
      }                                                                        \
    }                                                                          \
  } while (0)

// profile slots: 1..13 = forward operators; then the backward kernels in order
enum BackwardSlot {
  kB13Dropout = 14, kB12Grads, kB11Gelu, kB10Grads, kB98LayerNormDropout, kB7Grads, kB6DPd,
  kB6DV, kB54Softmax, kB3DQ, kB3DK, kB2Grads, kB2BiasGrad, kB1LayerNorm, kB6RowDot, kB654DScores,
  kOp36Fused, kB654DScoresFused, kB6DVFused, kNumSlots
};
static_assert(kNumSlots <= LYNX_PROFILE_SLOTS, "profile slots");
static_assert(LYNX_STATIC_WORKSPACE_BYTES == lynx::kStaticWorkspaceBytes, "header and library agree on the block size");
const char* const kSlotNames[kNumSlots] = {
    "", "op1_layernorm1", "op2_qkv_gemm", "op3_scores", "op4_softmax_dropout", "op5_attn_dropout",
    "op6_context", "op7_attn_proj_gemm", "op8_bias_dropout_add1", "op9_layernorm2", "op10_fc1_gemm",
    "op11_gelu", "op12_fc2_gemm", "op13_bias_dropout_add2", "b13_dropout_bwd",
    "b12_fc2_dgrad_wgrad", "b11_gelu_bwd", "b10_fc1_dgrad_wgrad",
    "b98_layernorm2_dropout_bwd", "b7_proj_dgrad_wgrad", "b6_dpd", "b6_dv", "b54_softmax_dropout_bwd", "b3_dq",
    "b3_dk", "b2_qkv_dgrad_wgrad", "b2_bias_grad", "b1_layernorm1_bwd", "b6_rowdot", "b654_dscores",
    "op3456_attention_fused", "b654_dscores_fused", "b6_dv_fused"};

char* act_ptr(const Ctx& cx, int i) {
  if (i == 0) return const_cast<char*>(static_cast<const char*>(cx.L->x));
  if (i == 13) return static_cast<char*>(cx.L->out);
  return cx.L->base + cx.bk->off[i];
}
float* stats_ptr(const Ctx& cx, int i) {  // mean[T], rstd[T] behind Y1 / Y2
  return reinterpret_cast<float*>(act_ptr(cx, i) + static_cast<size_t>(cx.L->D.T) * cx.L->D.h * cx.L->D.e);
}
float* attn_stats_ptr(const Ctx& cx) {  // (max, 1 / sum)[b a s] behind C
  return reinterpret_cast<float*>(act_ptr(cx, 6) + static_cast<size_t>(cx.L->D.T) * cx.L->D.p * cx.L->D.e);
}

lynx_status alloc_act(Ctx& cx, int i) {
  if (i == 13) { cx.bk->live[13] = true; return LYNX_OK; }
  size_t off;
  if (!cx.bk->arena.alloc(act_bytes(cx.L->D, i), &off)) return LYNX_ERR_OOM;
  cx.bk->off[i] = off;
  cx.bk->live[i] = true;
  return LYNX_OK;
}
void free_act(Ctx& cx, int i) {
  if (i < 1 || i > 12 || !cx.bk->live[i]) return;
  cx.bk->arena.release(cx.bk->off[i]);
  cx.bk->live[i] = false;
}

struct Temp {  // transient workspace block
  size_t off = 0;
  bool held = false;
};
lynx_status alloc_temp(Ctx& cx, size_t bytes, Temp* t) {
  if (!cx.bk->arena.alloc(bytes, &t->off)) return LYNX_ERR_OOM;
  t->held = true;
  return LYNX_OK;
}
void free_temp(Ctx& cx, Temp* t) {
  if (t->held) cx.bk->arena.release(t->off);
  t->held = false;
}
char* temp_ptr(const Ctx& cx, const Temp& t) { return cx.L->base + t.off; }

// Gradients a tap may name, and their sizes: those every kernel path materialises.
constexpr uint32_t kTappable = (1u << 12) | (1u << 10) | (1u << 9) | (1u << 8) | (1u << 7) | (1u << 6) |
                               (1u << 3) | (1u << 2) | (1u << 1);
size_t tap_bytes(const Dims& D, int i) {
  if (i == 1 || i == 9) return static_cast<size_t>(D.T) * D.h * D.e;  // without the statistics
  if (i == 6) return static_cast<size_t>(D.T) * D.p * D.e;
  return act_bytes(D, i);
}
lynx_status tap(Ctx& cx, int i, const void* grad) {
  void* dst = cx.L->grad_tap[i];
  if (!cx.launch || dst == nullptr) return LYNX_OK;
  const hipError_t e = hipMemcpyAsync(dst, grad, tap_bytes(cx.L->D, i), hipMemcpyDeviceToDevice, cx.st);
  if (e != hipSuccess) { cx.hip = e; return LYNX_ERR_HIP; }
  return LYNX_OK;
}

lynx::DropoutParams dropout_params(const lynx_layer_s* L) {
  return lynx::DropoutParams{L->cfg.seed, L->step, L->cfg.layer_id, L->cfg.dropout_p};
}
lynx::AttnShape attn_shape(const lynx_layer_s* L) {
  return lynx::AttnShape{L->D.b, L->D.a, L->D.s, L->D.a * L->cfg.tp_size, L->cfg.tp_rank * L->D.a};
}

// ---- matrix-product descriptors -------------------------------------------
// C[M, N] = A[M, K] * W[N, K]^T (+ bias): forward of a linear layer.
GemmDesc linear_fwd(const void* A, const void* W, const void* bias, void* C, int M, int N, int K) {
  GemmDesc g{};
  g.M = M; g.N = N; g.K = K;
  g.A = A; g.a_sm = K; g.a_sk = 1;
  g.B = W; g.b_sk = 1; g.b_sn = K;
  g.C = C; g.c_sm = N;
  g.bias = bias; g.nz1 = g.nz2 = 1; g.causal = lynx::kCausalNone;
  return g;
}
// dA[M, K] = dC[M, N] * W[N, K]: input gradient.
GemmDesc linear_dgrad(const void* dC, const void* W, void* dA, int M, int N, int K) {
  GemmDesc g{};
  g.M = M; g.N = K; g.K = N;
  g.A = dC; g.a_sm = N; g.a_sk = 1;
  g.B = W; g.b_sk = K; g.b_sn = 1;
  g.C = dA; g.c_sm = K;
  g.nz1 = g.nz2 = 1; g.causal = lynx::kCausalNone;
  return g;
}
// dW[N, K] = dC[M, N]^T * A[M, K]: weight gradient (contraction over tokens).
GemmDesc linear_wgrad(const void* dC, const void* A, void* dW, int M, int N, int K) {
  GemmDesc g{};
  g.M = N; g.N = K; g.K = M;
  g.A = dC; g.a_sm = 1; g.a_sk = N;
  g.B = A; g.b_sk = K; g.b_sn = 1;
  g.C = dW; g.c_sm = K;
  g.nz1 = g.nz2 = 1; g.causal = lynx::kCausalNone;
  return g;
}

// Batched attention products over (batch element, head).  `qkv` and `dqkv`
// are [T, 3p] with column blocks q | k | v; sq is a [b, a, s, s] tensor.
const char* col_block(const void* base, const Dims& D, int which) {
  return static_cast<const char*>(base) + static_cast<size_t>(which) * D.p * D.e;
}
void set_batch(GemmDesc& g, const Dims& D) { g.nz1 = D.b; g.nz2 = D.a; }

// out[i, j] = sum_dd x[i, dd] * y[j, dd], j <= i   (S = Q K^T, dPd = dC V^T)
GemmDesc attn_outer(const void* x, long long ldx, const void* y, long long ldy, void* sq,
                    const Dims& D) {
  GemmDesc g{};
  g.M = D.s; g.N = D.s; g.K = D.d;
  g.A = x; g.a_sm = ldx; g.a_sk = 1; g.a_sz1 = static_cast<long long>(D.s) * ldx; g.a_sz2 = D.d;
  g.B = y; g.b_sk = 1; g.b_sn = ldy; g.b_sz1 = static_cast<long long>(D.s) * ldy; g.b_sz2 = D.d;
  g.C = sq; g.c_sm = D.s; g.c_sz1 = static_cast<long long>(D.a) * D.s * D.s;
  g.c_sz2 = static_cast<long long>(D.s) * D.s;
  set_batch(g, D);
  g.causal = lynx::kCausalOutLower;
  return g;
}
// out[i, dd] = sum_{j <= i} sq[i, j] * y[j, dd]   (C = Pd V, dQ = dS K)
GemmDesc attn_rows(const void* sq, const void* y, long long ldy, void* out, long long ldo,
                   const Dims& D) {
  GemmDesc g{};
  g.M = D.s; g.N = D.d; g.K = D.s;
  g.A = sq; g.a_sm = D.s; g.a_sk = 1; g.a_sz1 = static_cast<long long>(D.a) * D.s * D.s;
  g.a_sz2 = static_cast<long long>(D.s) * D.s;
  g.B = y; g.b_sk = ldy; g.b_sn = 1; g.b_sz1 = static_cast<long long>(D.s) * ldy; g.b_sz2 = D.d;
  g.C = out; g.c_sm = ldo; g.c_sz1 = static_cast<long long>(D.s) * ldo; g.c_sz2 = D.d;
  set_batch(g, D);
  g.causal = lynx::kCausalKLeM;
  return g;
}
// out[j, dd] = sum_{i >= j} sq[i, j] * y[i, dd]   (dV = Pd^T dC, dK = dS^T Q)
GemmDesc attn_cols(const void* sq, const void* y, long long ldy, void* out, long long ldo,
                   const Dims& D) {
  GemmDesc g{};
  g.M = D.s; g.N = D.d; g.K = D.s;
  g.A = sq; g.a_sm = 1; g.a_sk = D.s; g.a_sz1 = static_cast<long long>(D.a) * D.s * D.s;
  g.a_sz2 = static_cast<long long>(D.s) * D.s;
  g.B = y; g.b_sk = ldy; g.b_sn = 1; g.b_sz1 = static_cast<long long>(D.s) * ldy; g.b_sz2 = D.d;
  g.C = out; g.c_sm = ldo; g.c_sz1 = static_cast<long long>(D.s) * ldo; g.c_sz2 = D.d;
  set_batch(g, D);
  g.causal = lynx::kCausalKGeM;
  return g;
}

// ---- forward operators ------------------------------------------------------
// Runs OP_i; its inputs are resident.  `fuse_dropout`: OP4 also emits Pd
// (then OP5 is skipped by the caller); `write_p`: whether OP4 stores P.
lynx_status run_op(Ctx& cx, int i, bool fuse_dropout = false, bool write_p = true) {
  lynx_layer_s* L = cx.L;
  const Dims& D = L->D;
  const lynx_params& w = L->params;
  const int dt = D.dtype;
  if (i == 4 && !write_p) {
    // P itself is not wanted: only Pd is produced
    LYNX_TRY(alloc_act(cx, 5));
    LYNX_LAUNCH(cx, i, lynx::softmax_dropout_fwd(dt, act_ptr(cx, 3), nullptr, act_ptr(cx, 5),
                                              attn_shape(L), 1.0f / sqrtf(static_cast<float>(D.d)),
                                              dropout_params(L), cx.st));
    return LYNX_OK;
  }
  LYNX_TRY(alloc_act(cx, i));
  switch (i) {
    case 1:
      LYNX_LAUNCH(cx, i, lynx::layernorm_fwd(dt, act_ptr(cx, 0), w.g1, w.be1, act_ptr(cx, 1),
                                          stats_ptr(cx, 1), stats_ptr(cx, 1) + D.T, D.T, D.h,
                                          L->cfg.ln_eps, cx.st));
      break;
    case 2:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, linear_fwd(act_ptr(cx, 1), w.wqkv, w.bqkv, act_ptr(cx, 2), D.T,
                                                3 * D.p, D.h), cx.st));
      break;
    case 3:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, attn_outer(col_block(act_ptr(cx, 2), D, 0), 3 * D.p,
                                                col_block(act_ptr(cx, 2), D, 1), 3 * D.p,
                                                act_ptr(cx, 3), D), cx.st));
      break;
    case 4: {
      void* pd = nullptr;
      if (fuse_dropout) {
        LYNX_TRY(alloc_act(cx, 5));
        pd = act_ptr(cx, 5);
      }
      LYNX_LAUNCH(cx, i, lynx::softmax_dropout_fwd(dt, act_ptr(cx, 3), act_ptr(cx, 4), pd,
                                                attn_shape(L), 1.0f / sqrtf(static_cast<float>(D.d)),
                                                dropout_params(L), cx.st));
      break;
    }
    case 5:
      LYNX_LAUNCH(cx, i, lynx::attn_dropout_fwd(dt, act_ptr(cx, 4), act_ptr(cx, 5), attn_shape(L),
                                             dropout_params(L), cx.st));
      break;
    case 6:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, attn_rows(act_ptr(cx, 5), col_block(act_ptr(cx, 2), D, 2),
                                               3 * D.p, act_ptr(cx, 6), D.p, D), cx.st));
      break;
    case 7:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, linear_fwd(act_ptr(cx, 6), w.wo, nullptr, act_ptr(cx, 7), D.T,
                                                D.h, D.p), cx.st));
      break;
    case 8:
      LYNX_LAUNCH(cx, i, lynx::bias_dropout_add_fwd(dt, act_ptr(cx, 7), w.bo, act_ptr(cx, 0),
                                                 act_ptr(cx, 8), D.T, D.h, 1, dropout_params(L),
                                                 cx.st));
      break;
    case 9:
      LYNX_LAUNCH(cx, i, lynx::layernorm_fwd(dt, act_ptr(cx, 8), w.g2, w.be2, act_ptr(cx, 9),
                                          stats_ptr(cx, 9), stats_ptr(cx, 9) + D.T, D.T, D.h,
                                          L->cfg.ln_eps, cx.st));
      break;
    case 10:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, linear_fwd(act_ptr(cx, 9), w.w1, w.b1, act_ptr(cx, 10), D.T,
                                                D.f, D.h), cx.st));
      break;
    case 11:
      LYNX_LAUNCH(cx, i, lynx::gelu_fwd(dt, act_ptr(cx, 10), act_ptr(cx, 11),
                                     static_cast<size_t>(D.T) * D.f, cx.st));
      break;
    case 12:
      LYNX_LAUNCH(cx, i, lynx::gemm(dt, linear_fwd(act_ptr(cx, 11), w.w2, nullptr, act_ptr(cx, 12),
                                                D.T, D.h, D.f), cx.st));
      break;
    case 13:
      LYNX_LAUNCH(cx, i, lynx::bias_dropout_add_fwd(dt, act_ptr(cx, 12), w.b2, act_ptr(cx, 8),
                                                 act_ptr(cx, 13), D.T, D.h, 2, dropout_params(L),
                                                 cx.st));
      break;
    default:
      return LYNX_ERR_INVALID_ARG;
  }
  return LYNX_OK;
}

// OP7 + OP8 (or OP12 + OP13) as one launch: the product of operator `lin` is rounded as
// it would be stored, and the store pass of the matrix-product kernel applies bias,
// dropout and residual to it, so the operator that would read it back never runs.  The
// product itself is kept (written as well) only if the policy retains it.  Same bits as the
// two operators run one after the other.
GemmDesc fused_linear_desc(Ctx& cx, int lin, bool keep_product) {
  lynx_layer_s* L = cx.L;
  const Dims& D = L->D;
  const lynx_params& w = L->params;
  const bool first = lin == 7;
  GemmDesc g = first ? linear_fwd(act_ptr(cx, 6), w.wo, nullptr, nullptr, D.T, D.h, D.p)
                     : linear_fwd(act_ptr(cx, 11), w.w2, nullptr, nullptr, D.T, D.h, D.f);
  g.C = cx.bk->live[lin + 1] ? act_ptr(cx, lin + 1) : nullptr;
  g.epi.kind = lynx::kEpiBiasDropoutAdd;
  g.epi.aux = first ? act_ptr(cx, 0) : act_ptr(cx, 8);
  g.epi.aux_ld = D.h;
  g.epi.vec = first ? w.bo : w.b2;
  g.epi.plain = keep_product ? act_ptr(cx, lin) : nullptr;
  g.epi.site = first ? 1 : 2;
  g.epi.dp = dropout_params(L);
  return g;
}
bool can_fuse_linear(const lynx_layer_s* L, int lin) {
  const Dims& D = L->D;
  // shapes only (pointers are 256-byte aligned arena blocks or checked caller buffers)
  GemmDesc g = linear_fwd(reinterpret_cast<const void*>(256), reinterpret_cast<const void*>(256), nullptr,
                          reinterpret_cast<void*>(256), D.T, D.h, lin == 7 ? D.p : D.f);
  g.epi.kind = lynx::kEpiBiasDropoutAdd;
  g.epi.aux = reinterpret_cast<const void*>(256);
  g.epi.aux_ld = D.h;
  g.epi.vec = reinterpret_cast<const void*>(256);
  return lynx::gemm_mfma_supported(D.dtype, g);
}
lynx_status run_fused_linear(Ctx& cx, int lin) {
  const bool keep_product = (cx.bk->retain >> lin) & 1u;
  if (keep_product) LYNX_TRY(alloc_act(cx, lin));
  LYNX_TRY(alloc_act(cx, lin + 1));
  LYNX_LAUNCH(cx, lin, lynx::gemm(cx.L->D.dtype, fused_linear_desc(cx, lin, keep_product), cx.st));
  return LYNX_OK;
}

// Operators 3-6 as one launch (attn_fused.hip): C and its row statistics from QKV.
lynx_status run_fused_attention(Ctx& cx) {
  lynx_layer_s* L = cx.L;
  const Dims& D = L->D;
  LYNX_TRY(alloc_act(cx, 6));
  LYNX_LAUNCH(cx, kOp36Fused, lynx::attn_fused_fwd(act_ptr(cx, 2), 3 * D.p, act_ptr(cx, 6), D.p, attn_stats_ptr(cx),
                                          attn_shape(L), D.d, 1.0f / sqrtf(static_cast<float>(D.d)),
                                          dropout_params(L), cx.st));
  return LYNX_OK;
}

lynx_status forward_pass(Ctx& cx, uint32_t retain) {
  Book& bk = *cx.bk;
  bk.retain = (retain & 0x3FFFu) | kCallerOwned;
  bk.live[0] = true;
  bk.fused_attn = (cx.L->cfg.flags & LYNX_FLAG_FUSED_ATTENTION) && !(bk.retain & 0x38u) &&
                  lynx::attn_fused_supported(cx.L->D.dtype, cx.L->D.s, cx.L->D.d);
  for (int i = 1; i <= kNumOps; ++i) {
    if (i == 5) continue;  // emitted by OP4's kernel
    int done = i;
    if (bk.fused_attn && (i == 3 || i == 4)) continue;
    if (bk.fused_attn && i == 6) {
      LYNX_TRY(run_fused_attention(cx));
    } else if (i == 4) {
      LYNX_TRY(run_op(cx, 4, /*fuse_dropout=*/true, /*write_p=*/(bk.retain >> 4) & 1u));
      done = 5;  // OP4's launch covers OP5
    } else if ((i == 7 || i == 12) && can_fuse_linear(cx.L, i)) {
      LYNX_TRY(run_fused_linear(cx, i));
      done = ++i;  // the launch covers the bias + dropout + residual operator too
    } else {
      LYNX_TRY(run_op(cx, i));
    }
    for (int j = 1; j <= 12; ++j)
      if (bk.live[j] && kLastForwardUse[j] <= done && !((bk.retain >> j) & 1u)) free_act(cx, j);
  }
  bk.state = 1;
  return LYNX_OK;
}

// Regenerated activations that backward never reads are dropped once every
// operator that consumes them has its output resident.
void release_stepping_stones(Ctx& cx) {
  Book& bk = *cx.bk;
  static const int stones[3] = {3, 7, 12};
  for (int j : stones) {
    if (!bk.live[j] || ((bk.retain >> j) & 1u)) continue;
    bool all = true;
    for (int op = 1; op <= kNumOps; ++op)
      for (int k = 0; k < 3 && kParents[op][k] >= 0; ++k)
        if (kParents[op][k] == j && !bk.live[op]) all = false;
    if (all) free_act(cx, j);
  }
}

// The operator graph as this call sees it.  With the attention fused (Book::fused_attn)
// operators 3-5 do not exist: operator 6 reads QKV alone and backward reads C with its row
// statistics instead of P and Pd.
int parent_of(const Book& bk, int op, int k) {
  if (bk.fused_attn && op == 6) return k == 0 ? 2 : -1;
  return k < 3 ? kParents[op][k] : -1;
}
uint32_t backward_needs(const Book& bk) {
  return bk.fused_attn ? (kBackwardNeeds & ~((1u << 4) | (1u << 5))) : kBackwardNeeds;
}

uint32_t missing_closure(const Book& bk) {
  uint32_t todo = 0;
  std::vector<int> stack;
  const uint32_t needs = backward_needs(bk);
  for (int i = 0; i < kNumAct; ++i)
    if (((needs >> i) & 1u) && !bk.live[i]) stack.push_back(i);
  while (!stack.empty()) {
    const int i = stack.back();
    stack.pop_back();
    if ((todo >> i) & 1u) continue;
    todo |= 1u << i;
    for (int k = 0; k < 3 && parent_of(bk, i, k) >= 0; ++k) {
      const int j = parent_of(bk, i, k);
      if (!bk.live[j] && !((todo >> j) & 1u)) stack.push_back(j);
    }
  }
  return todo;
}

lynx_status recompute_pass(Ctx& cx, uint32_t segment) {
  Book& bk = *cx.bk;
  if (segment == LYNX_SEG_ALL_MISSING) segment = missing_closure(bk);
  if (segment & ~0x3FFFu) return LYNX_ERR_INVALID_ARG;
  if (bk.fused_attn) segment &= ~0x38u;  // operators 3-5 do not exist in this mode: naming them is a no-op
  // dependency rule: every input stored or produced earlier in the segment
  {
    bool have[kNumAct];
    for (int i = 0; i < kNumAct; ++i) have[i] = bk.live[i];
    for (int i = 1; i <= kNumOps; ++i) {
      if (!((segment >> i) & 1u) || have[i]) continue;
      for (int k = 0; k < 3 && parent_of(bk, i, k) >= 0; ++k)
        if (!have[parent_of(bk, i, k)]) return LYNX_ERR_DEPENDENCY;
      have[i] = true;
    }
  }
  for (int i = 1; i <= kNumOps; ++i) {
    if (!((segment >> i) & 1u) || bk.live[i]) continue;
    if (bk.fused_attn && i == 6) {
      LYNX_TRY(run_fused_attention(cx));
    } else if (i == 4 && ((segment >> 5) & 1u) && !bk.live[5]) {
      LYNX_TRY(run_op(cx, 4, /*fuse_dropout=*/true));
    } else if ((i == 7 || i == 12) && ((segment >> (i + 1)) & 1u) && !bk.live[i + 1] &&
               can_fuse_linear(cx.L, i)) {
      LYNX_TRY(run_fused_linear(cx, i));
      ++i;
    } else {
      LYNX_TRY(run_op(cx, i));
    }
    release_stepping_stones(cx);
  }
  return LYNX_OK;
}

// ---- backward ---------------------------------------------------------------
lynx_status backward_pass(Ctx& cx, const void* d_out, void* d_x, const lynx_grads* gr) {
  lynx_layer_s* L = cx.L;
  const Dims& D = L->D;
  const lynx_params& w = L->params;
  const int dt = D.dtype;
  const size_t e = D.e;
  LYNX_TRY(recompute_pass(cx, LYNX_SEG_ALL_MISSING));

  const int widest = D.h > 3 * D.p ? (D.h > D.f ? D.h : D.f) : (3 * D.p > D.f ? 3 * D.p : D.f);
  size_t scratch_bytes = lynx::colsum_scratch_bytes(D.T, widest);
  const size_t ln_bytes = lynx::layernorm_bwd_scratch_bytes(D.T, D.h);
  if (ln_bytes > scratch_bytes) scratch_bytes = ln_bytes;
  {  // fp32 partial sums of weight gradients that are cut into K ranges
    const int lin[4][2] = {{D.h, D.f}, {D.f, D.h}, {D.h, D.p}, {3 * D.p, D.h}};  // {outputs, inputs}
    for (const auto& nk : lin) {
      const size_t b = lynx::gemm_pair_scratch_bytes(dt, linear_dgrad(nullptr, nullptr, nullptr, D.T, nk[0], nk[1]),
                                                     linear_wgrad(nullptr, nullptr, nullptr, D.T, nk[0], nk[1]));
      if (b > scratch_bytes) scratch_bytes = b;
    }
  }
  Temp scratch, t_dv2, t_dg, t_du, t_dy2, t_dx2, t_do, t_dc, t_dpd, t_dqkv, t_dy1;
  LYNX_TRY(alloc_temp(cx, scratch_bytes, &scratch));
  float* scr = reinterpret_cast<float*>(temp_ptr(cx, scratch));
  const size_t th = static_cast<size_t>(D.T) * D.h * e, tf = static_cast<size_t>(D.T) * D.f * e;

  // B13: OUT = X2 + keep2 (V2 + b2) c
  LYNX_TRY(alloc_temp(cx, th, &t_dv2));
  LYNX_LAUNCH(cx, kB13Dropout, lynx::dropout_bwd(dt, d_out, temp_ptr(cx, t_dv2), gr->b2, scr, D.T, D.h, 2,
                                    dropout_params(L), cx.st));
  LYNX_TRY(tap(cx, 12, temp_ptr(cx, t_dv2)));
  // B12: V2 = G W2^T, and B11: G = gelu(U).  When the matrix-core pair launch applies, the
  // store pass of the input gradient multiplies by gelu'(U) and sums the columns (the FC1
  // bias gradient), so dG is never written and the GeLU backward never runs as a kernel.
  LYNX_TRY(alloc_temp(cx, tf, &t_du));
  {
    GemmDesc dg = linear_dgrad(temp_ptr(cx, t_dv2), w.w2, temp_ptr(cx, t_du), D.T, D.h, D.f);
    const GemmDesc wg = linear_wgrad(temp_ptr(cx, t_dv2), act_ptr(cx, 11), gr->w2, D.T, D.h, D.f);
    Temp t_colsum;
    LYNX_TRY(alloc_temp(cx, lynx::gemm_colsum_partial_bytes(D.T, D.f), &t_colsum));
    dg.epi.kind = lynx::kEpiGeluBwd;
    dg.epi.aux = act_ptr(cx, 10);
    dg.epi.aux_ld = D.f;
    dg.epi.colsum_partial = reinterpret_cast<float*>(temp_ptr(cx, t_colsum));
    dg.epi.colsum_out = gr->b1;
    if (lynx::gemm_mfma_pair_supported(dt, dg, wg)) {
      LYNX_LAUNCH(cx, kB12Grads, lynx::gemm_mfma_pair(dg, wg, scr, scratch_bytes, cx.st));
      free_temp(cx, &t_colsum);
      free_temp(cx, &t_dv2);
      free_act(cx, 11);
    } else {
      free_temp(cx, &t_colsum);
      dg.epi = lynx::GemmEpilogue{};
      LYNX_TRY(alloc_temp(cx, tf, &t_dg));
      dg.C = temp_ptr(cx, t_dg);
      LYNX_LAUNCH(cx, kB12Grads, lynx::gemm_pair(dt, dg, wg, scr, scratch_bytes, cx.st));
      free_temp(cx, &t_dv2);
      free_act(cx, 11);
      LYNX_LAUNCH(cx, kB11Gelu, lynx::gelu_bwd(dt, temp_ptr(cx, t_dg), act_ptr(cx, 10), temp_ptr(cx, t_du),
                                               gr->b1, scr, D.T, D.f, cx.st));
      free_temp(cx, &t_dg);
    }
  }
  free_act(cx, 10);
  LYNX_TRY(tap(cx, 10, temp_ptr(cx, t_du)));
  // B10: U = Y2 W1^T + b1
  LYNX_TRY(alloc_temp(cx, th, &t_dy2));
  LYNX_LAUNCH(cx, kB10Grads, lynx::gemm_pair(dt, linear_dgrad(temp_ptr(cx, t_du), w.w1, temp_ptr(cx, t_dy2), D.T, D.f, D.h),
                                                  linear_wgrad(temp_ptr(cx, t_du), act_ptr(cx, 9), gr->w1, D.T, D.f, D.h), scr, scratch_bytes, cx.st));
  free_temp(cx, &t_du);
  LYNX_TRY(tap(cx, 9, temp_ptr(cx, t_dy2)));
  // B9: Y2 = LN2(X2); dX2 = dOUT + dLN.  B8 in the same pass: X2 = X + keep1 (O + bo) c,
  // so dO = keep1 c dX2 and dbo = its column sums
  LYNX_TRY(alloc_temp(cx, th, &t_dx2));
  LYNX_TRY(alloc_temp(cx, th, &t_do));
  LYNX_LAUNCH(cx, kB98LayerNormDropout,
              lynx::layernorm_bwd_dropout_bwd(dt, temp_ptr(cx, t_dy2), act_ptr(cx, 8), stats_ptr(cx, 9),
                                              stats_ptr(cx, 9) + D.T, w.g2, d_out, temp_ptr(cx, t_dx2), gr->g2,
                                              gr->be2, temp_ptr(cx, t_do), gr->bo, scr, D.T, D.h, 1,
                                              dropout_params(L), cx.st));
  LYNX_TRY(tap(cx, 8, temp_ptr(cx, t_dx2)));
  LYNX_TRY(tap(cx, 7, temp_ptr(cx, t_do)));
  free_temp(cx, &t_dy2);
  free_act(cx, 9);
  free_act(cx, 8);
  // B7: O = C Wo^T
  LYNX_TRY(alloc_temp(cx, static_cast<size_t>(D.T) * D.p * e, &t_dc));
  LYNX_LAUNCH(cx, kB7Grads, lynx::gemm_pair(dt, linear_dgrad(temp_ptr(cx, t_do), w.wo, temp_ptr(cx, t_dc), D.T, D.h, D.p),
                                                  linear_wgrad(temp_ptr(cx, t_do), act_ptr(cx, 6), gr->wo, D.T, D.h, D.p), scr, scratch_bytes, cx.st));
  free_temp(cx, &t_do);
  LYNX_TRY(tap(cx, 6, temp_ptr(cx, t_dc)));
  // B6: C = Pd V (C itself is read once more below, for the row dot products)
  LYNX_TRY(alloc_temp(cx, D.ss * e, &t_dpd));
  LYNX_TRY(alloc_temp(cx, static_cast<size_t>(D.T) * 3 * D.p * e, &t_dqkv));
  char* dqkv = temp_ptr(cx, t_dqkv);
  const char* qkv = act_ptr(cx, 2);
  // dPd = dC V^T, then B5 + B4: Pd = keep0 P c, P = softmax(S / sqrt(d)).  Where the row-block
  // kernel applies, the store pass of the product forms dS directly (dPd is never written);
  // the row dot products sum_j dP_ij P_ij it needs equal sum_dd dC[i, dd] C[i, dd] and come
  // from a small kernel over dC and C.  Otherwise dPd is stored and dS overwrites it.
  GemmDesc dpd = attn_outer(temp_ptr(cx, t_dc), D.p, col_block(qkv, D, 2), 3 * D.p, temp_ptr(cx, t_dpd), D);
  Temp t_rowdot;
  LYNX_TRY(alloc_temp(cx, static_cast<size_t>(D.b) * D.a * D.s * sizeof(float), &t_rowdot));
  dpd.epi.kind = lynx::kEpiSoftmaxBwd;
  dpd.epi.aux = act_ptr(cx, 4);
  dpd.epi.aux_ld = D.s;
  dpd.epi.rowdot = reinterpret_cast<const float*>(temp_ptr(cx, t_rowdot));
  dpd.epi.scale = 1.0f / sqrtf(static_cast<float>(D.d));
  dpd.epi.dp = dropout_params(L);
  dpd.epi.global_heads = D.a * L->cfg.tp_size;
  dpd.epi.head0 = L->cfg.tp_rank * D.a;
  const bool fused_ds = lynx::gemm_mfma_supported(dt, dpd);
  // dV = Pd^T dC.  With the one-pass dS kernel it goes first, so that dQ and dK read dS right
  // after it is written, while much of it is still in the caches (measured: dQ 0.070 -> 0.05x ms).
  const bool dv_first = fused_ds && !cx.bk->fused_attn;
  auto launch_dv = [&]() -> lynx_status {
    LYNX_LAUNCH(cx, kB6DV, lynx::gemm(dt, attn_cols(act_ptr(cx, 5), temp_ptr(cx, t_dc), D.p,
                                             const_cast<char*>(col_block(dqkv, D, 2)), 3 * D.p, D),
                               cx.st));
    return LYNX_OK;
  };
  if (dv_first) {
    LYNX_TRY(launch_dv());
    free_act(cx, 5);
  }
  if (cx.bk->fused_attn) {
    // neither P nor Pd exists: both kernels rebuild them from QKV and the row statistics of C
    float* rowdot = reinterpret_cast<float*>(temp_ptr(cx, t_rowdot));
    LYNX_LAUNCH(cx, kB6RowDot, lynx::attn_rowdot(dt, temp_ptr(cx, t_dc), act_ptr(cx, 6), rowdot, D.b, D.a, D.s, D.d,
                                                 D.p, cx.st));
    LYNX_LAUNCH(cx, kB654DScoresFused, lynx::attn_fused_bwd_ds(qkv, 3 * D.p, temp_ptr(cx, t_dc), D.p, attn_stats_ptr(cx),
                                                          rowdot, temp_ptr(cx, t_dpd), attn_shape(L), D.d,
                                                          dpd.epi.scale, dropout_params(L), cx.st));
  } else if (fused_ds) {
    LYNX_LAUNCH(cx, kB6RowDot, lynx::attn_rowdot(dt, temp_ptr(cx, t_dc), act_ptr(cx, 6),
                                                 reinterpret_cast<float*>(temp_ptr(cx, t_rowdot)), D.b, D.a, D.s,
                                                 D.d, D.p, cx.st));
    LYNX_LAUNCH(cx, kB654DScores, lynx::gemm_mfma(dpd, cx.st));
  } else {
    dpd.epi = lynx::GemmEpilogue{};
    LYNX_LAUNCH(cx, kB6DPd, lynx::gemm(dt, dpd, cx.st));
  }
  free_temp(cx, &t_rowdot);
  if (cx.bk->fused_attn) {
    LYNX_LAUNCH(cx, kB6DVFused, lynx::attn_fused_bwd_dv(qkv, 3 * D.p, temp_ptr(cx, t_dc), D.p, attn_stats_ptr(cx), dqkv,
                                                   3 * D.p, attn_shape(L), D.d, 1.0f / sqrtf(static_cast<float>(D.d)),
                                                   dropout_params(L), cx.st));
  } else if (!dv_first) {
    LYNX_TRY(launch_dv());
  }
  free_temp(cx, &t_dc);
  free_act(cx, 5);
  free_act(cx, 6);
  if (!fused_ds && !cx.bk->fused_attn) {
    LYNX_LAUNCH(cx, kB54Softmax, lynx::softmax_dropout_bwd(dt, temp_ptr(cx, t_dpd), act_ptr(cx, 4),
                                              temp_ptr(cx, t_dpd), attn_shape(L),
                                              1.0f / sqrtf(static_cast<float>(D.d)), dropout_params(L),
                                              cx.st));
  }
  free_act(cx, 4);
  LYNX_TRY(tap(cx, 3, temp_ptr(cx, t_dpd)));
  // B3: S = Q K^T
  LYNX_LAUNCH(cx, kB3DQ, lynx::gemm(dt, attn_rows(temp_ptr(cx, t_dpd), col_block(qkv, D, 1), 3 * D.p,
                                           const_cast<char*>(col_block(dqkv, D, 0)), 3 * D.p, D),
                             cx.st));
  LYNX_LAUNCH(cx, kB3DK, lynx::gemm(dt, attn_cols(temp_ptr(cx, t_dpd), col_block(qkv, D, 0), 3 * D.p,
                                           const_cast<char*>(col_block(dqkv, D, 1)), 3 * D.p, D),
                             cx.st));
  free_temp(cx, &t_dpd);
  free_act(cx, 3);
  LYNX_TRY(tap(cx, 2, dqkv));
  // B2: QKV = Y1 Wqkv^T + bqkv
  LYNX_TRY(alloc_temp(cx, th, &t_dy1));
  LYNX_LAUNCH(cx, kB2Grads, lynx::gemm_pair(dt, linear_dgrad(dqkv, w.wqkv, temp_ptr(cx, t_dy1), D.T, 3 * D.p, D.h),
                                                  linear_wgrad(dqkv, act_ptr(cx, 1), gr->wqkv, D.T, 3 * D.p, D.h), scr, scratch_bytes, cx.st));
  LYNX_LAUNCH(cx, kB2BiasGrad, lynx::column_sum(dt, dqkv, gr->bqkv, scr, D.T, 3 * D.p, cx.st));
  free_temp(cx, &t_dqkv);
  free_act(cx, 2);
  LYNX_TRY(tap(cx, 1, temp_ptr(cx, t_dy1)));
  // B1: Y1 = LN1(X); dX = dX2 + dLN
  LYNX_LAUNCH(cx, kB1LayerNorm, lynx::layernorm_bwd(dt, temp_ptr(cx, t_dy1), act_ptr(cx, 0), stats_ptr(cx, 1),
                                      stats_ptr(cx, 1) + D.T, w.g1, temp_ptr(cx, t_dx2), d_x, gr->g1,
                                      gr->be1, scr, D.T, D.h, cx.st));
  free_temp(cx, &t_dy1);
  free_temp(cx, &t_dx2);
  free_temp(cx, &scratch);
  for (int i = 1; i <= 12; ++i) free_act(cx, i);
  for (int i = 0; i < kNumAct; ++i) cx.bk->live[i] = false;
  cx.bk->state = 0;
  return LYNX_OK;
}

bool aligned16(const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool grads_ok(const lynx_grads* g) {
  if (g == nullptr) return false;
  const void* const* p = reinterpret_cast<const void* const*>(g);
  for (int i = 0; i < 12; ++i)
    if (!aligned16(p[i])) return false;
  return true;
}

// Rehearse on a copy, then run for real.
template <typename F>
lynx_status two_pass(lynx_layer_s* L, hipStream_t st, F&& body) {
  Book copy = L->book;
  Ctx rehearsal{L, &copy, false, st};
  LYNX_TRY(body(rehearsal));
  Ctx real{L, &L->book, !L->dry, st};
  return body(real);
}

}  // namespace

extern "C" {

size_t lynx_activation_bytes(const lynx_layer_config* cfg, int act_id) {
  Dims D;
  if (!make_dims(cfg, &D) || act_id < 0 || act_id >= kNumAct) return 0;
  return act_bytes(D, act_id);
}

lynx_status lynx_layer_create(const lynx_layer_config* cfg, void* workspace, size_t workspace_bytes,
                              lynx_layer_t* out_layer) {
  if (cfg == nullptr || out_layer == nullptr) return LYNX_ERR_INVALID_ARG;
  Dims D;
  if (!make_dims(cfg, &D)) return LYNX_ERR_SHAPE;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & (Arena::kAlign - 1)))
    return LYNX_ERR_INVALID_ARG;
  lynx_layer_s* L = new (std::nothrow) lynx_layer_s;
  if (L == nullptr) return LYNX_ERR_OOM;
  L->cfg = *cfg;
  L->D = D;
  L->base = static_cast<char*>(workspace);
  L->book.arena = Arena(workspace_bytes / Arena::kAlign * Arena::kAlign);
  *out_layer = L;
  return LYNX_OK;
}

lynx_status lynx_layer_create_static(const lynx_layer_config* cfg, lynx_layer_t* out_layer) {
  if (cfg == nullptr || out_layer == nullptr) return LYNX_ERR_INVALID_ARG;
  Dims D;
  if (!make_dims(cfg, &D)) return LYNX_ERR_SHAPE;
  // the leanest schedule of this shape (keep the input only) must fit the block
  const size_t least = lynx_workspace_bytes(cfg, LYNX_RETAIN_FULL_RECOMPUTE);
  if (least == 0 || least > lynx::kStaticWorkspaceBytes) return LYNX_ERR_OOM;
  lynx_layer_s* L = new (std::nothrow) lynx_layer_s;
  if (L == nullptr) return LYNX_ERR_OOM;
  void* base = nullptr;
  int device = -1;
  const hipError_t e = lynx::static_workspace_acquire(&base, &device);
  if (e != hipSuccess) {
    delete L;
    return e == hipErrorContextAlreadyInUse ? LYNX_ERR_STATE : LYNX_ERR_HIP;
  }
  L->cfg = *cfg;
  L->D = D;
  L->base = static_cast<char*>(base);
  L->book.arena = Arena(lynx::kStaticWorkspaceBytes);
  L->static_device = device;
  *out_layer = L;
  return LYNX_OK;
}

lynx_status lynx_layer_destroy(lynx_layer_t layer) {
  if (layer == nullptr) return LYNX_ERR_INVALID_ARG;
  (void)lynx_layer_set_profiling(layer, 0);
  if (layer->static_device >= 0) lynx::static_workspace_release(layer->static_device);
  delete layer;
  return LYNX_OK;
}

lynx_status lynx_layer_set_params(lynx_layer_t L, const lynx_params* params) {
  if (L == nullptr || params == nullptr) return LYNX_ERR_INVALID_ARG;
  const void* const* p = reinterpret_cast<const void* const*>(params);
  for (int i = 0; i < 12; ++i)
    if (!aligned16(p[i])) return LYNX_ERR_INVALID_ARG;
  L->params = *params;
  L->have_params = true;
  return LYNX_OK;
}

lynx_status lynx_layer_set_dry_run(lynx_layer_t L, int on) {
  if (L == nullptr) return LYNX_ERR_INVALID_ARG;
  L->dry = on != 0;
  return LYNX_OK;
}

lynx_status lynx_layer_forward(lynx_layer_t L, const void* x, void* out, uint32_t retain_mask,
                               uint64_t step, void* hip_stream) {
  if (L == nullptr || !aligned16(x) || !aligned16(out)) return LYNX_ERR_INVALID_ARG;
  if (retain_mask & ~0x3FFFu) return LYNX_ERR_INVALID_ARG;
  if (step >> 32) return LYNX_ERR_INVALID_ARG;
  if (!L->have_params || L->book.state != 0) return LYNX_ERR_STATE;
  const void* old_x = L->x;
  void* old_out = L->out;
  const uint64_t old_step = L->step;
  L->x = x; L->out = out; L->step = step;
  const lynx_status s = two_pass(L, static_cast<hipStream_t>(hip_stream),
                                 [&](Ctx& cx) { return forward_pass(cx, retain_mask); });
  if (s != LYNX_OK && s != LYNX_ERR_HIP) { L->x = old_x; L->out = old_out; L->step = old_step; }
  return s;
}

lynx_status lynx_recompute(lynx_layer_t L, uint32_t segment_mask, void* hip_stream) {
  if (L == nullptr) return LYNX_ERR_INVALID_ARG;
  if (L->book.state != 1) return LYNX_ERR_STATE;
  return two_pass(L, static_cast<hipStream_t>(hip_stream),
                  [&](Ctx& cx) { return recompute_pass(cx, segment_mask); });
}

lynx_status lynx_layer_backward(lynx_layer_t L, const void* d_out, void* d_x, const lynx_grads* grads,
                                void* hip_stream) {
  if (L == nullptr || !aligned16(d_out) || !aligned16(d_x) || !grads_ok(grads))
    return LYNX_ERR_INVALID_ARG;
  if (L->book.state != 1) return LYNX_ERR_STATE;
  return two_pass(L, static_cast<hipStream_t>(hip_stream),
                  [&](Ctx& cx) { return backward_pass(cx, d_out, d_x, grads); });
}

lynx_status lynx_layer_reset(lynx_layer_t L) {
  if (L == nullptr) return LYNX_ERR_INVALID_ARG;
  Ctx cx{L, &L->book, false, nullptr};
  for (int i = 1; i <= 12; ++i) free_act(cx, i);
  for (int i = 0; i < kNumAct; ++i) L->book.live[i] = false;
  L->book.state = 0;
  return LYNX_OK;
}

lynx_status lynx_layer_live_mask(lynx_layer_t L, uint32_t* live) {
  if (L == nullptr || live == nullptr) return LYNX_ERR_INVALID_ARG;
  uint32_t m = 0;
  for (int i = 0; i < kNumAct; ++i)
    if (L->book.live[i]) m |= 1u << i;
  *live = m;
  return LYNX_OK;
}

lynx_status lynx_layer_missing_mask(lynx_layer_t L, uint32_t* missing) {
  if (L == nullptr || missing == nullptr) return LYNX_ERR_INVALID_ARG;
  if (L->book.state != 1) return LYNX_ERR_STATE;
  *missing = missing_closure(L->book);
  return LYNX_OK;
}

lynx_status lynx_layer_live_bytes(lynx_layer_t L, size_t* bytes) {
  if (L == nullptr || bytes == nullptr) return LYNX_ERR_INVALID_ARG;
  size_t n = 0;
  for (int i = 1; i <= 12; ++i)
    if (L->book.live[i]) n += act_bytes(L->D, i);
  *bytes = n;
  return LYNX_OK;
}

lynx_status lynx_layer_peak_bytes(lynx_layer_t L, size_t* bytes) {
  if (L == nullptr || bytes == nullptr) return LYNX_ERR_INVALID_ARG;
  *bytes = L->book.arena.extent_peak();
  return LYNX_OK;
}

lynx_status lynx_layer_activation(lynx_layer_t L, int act_id, const void** device_ptr, size_t* bytes) {
  if (L == nullptr || device_ptr == nullptr || bytes == nullptr || act_id < 0 || act_id >= kNumAct)
    return LYNX_ERR_INVALID_ARG;
  *bytes = act_bytes(L->D, act_id);
  if (!L->book.live[act_id]) { *device_ptr = nullptr; return LYNX_OK; }
  Ctx cx{L, &L->book, false, nullptr};
  *device_ptr = act_ptr(cx, act_id);
  return LYNX_OK;
}

size_t lynx_workspace_bytes_for_schedule(const lynx_layer_config* cfg, uint32_t retain_mask,
                                         const uint32_t* phase_masks) {
  Dims D;
  if (!make_dims(cfg, &D) || (retain_mask & ~0x3FFFu)) return 0;
  lynx_layer_s L;
  L.cfg = *cfg;
  L.D = D;
  L.base = nullptr;
  L.book.arena = Arena(static_cast<size_t>(1) << 60);
  Ctx cx{&L, &L.book, false, nullptr};
  // Nothing is launched; the placeholders only have to look like what a real call passes
  // (non-null, aligned), so that the rehearsal takes the kernel path a real call takes.
  void* const fake = reinterpret_cast<void*>(static_cast<uintptr_t>(Arena::kAlign));
  const lynx_grads g{fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake};
  L.params = lynx_params{fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake};
  L.x = fake;
  L.out = fake;
  if (forward_pass(cx, retain_mask) != LYNX_OK) return 0;
  for (int t = 0; phase_masks != nullptr && t < 4; ++t)
    if (phase_masks[t] != 0 && recompute_pass(cx, phase_masks[t]) != LYNX_OK) return 0;
  if (backward_pass(cx, fake, fake, &g) != LYNX_OK) return 0;
  return L.book.arena.extent_peak();
}

size_t lynx_workspace_bytes(const lynx_layer_config* cfg, uint32_t retain_mask) {
  return lynx_workspace_bytes_for_schedule(cfg, retain_mask, nullptr);
}

lynx_status lynx_dropout_mask(const lynx_layer_config* cfg, uint64_t step, int site, uint8_t* out,
                              void* hip_stream) {
  Dims D;
  if (cfg == nullptr || out == nullptr || site < 0 || site > 2 || (step >> 32))
    return LYNX_ERR_INVALID_ARG;
  if (!make_dims(cfg, &D)) return LYNX_ERR_SHAPE;
  const lynx::DropoutParams dp{cfg->seed, step, cfg->layer_id, cfg->dropout_p};
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (site == 0)
    e = lynx::dropout_mask_attn(out, lynx::AttnShape{D.b, D.a, D.s, D.a * cfg->tp_size,
                                                     cfg->tp_rank * D.a}, dp, st);
  else
    e = lynx::dropout_mask_hidden(out, static_cast<size_t>(D.T) * D.h, site, dp, st);
  return e == hipSuccess ? LYNX_OK : LYNX_ERR_HIP;
}

lynx_status lynx_layer_set_gradient_tap(lynx_layer_t L, int act_id, void* device_dst) {
  if (L == nullptr || act_id < 0 || act_id >= kNumAct || !((kTappable >> act_id) & 1u))
    return LYNX_ERR_INVALID_ARG;
  if (device_dst != nullptr && !aligned16(device_dst)) return LYNX_ERR_INVALID_ARG;
  L->grad_tap[act_id] = device_dst;
  return LYNX_OK;
}

lynx_status lynx_layer_set_profiling(lynx_layer_t L, int on) {
  if (L == nullptr) return LYNX_ERR_INVALID_ARG;
  if ((on != 0) == L->profiling) return LYNX_OK;
  if (on) {
    for (int i = 0; i < LYNX_PROFILE_SLOTS; ++i) {
      if (hipEventCreate(&L->ev_begin[i]) != hipSuccess || hipEventCreate(&L->ev_end[i]) != hipSuccess)
        return LYNX_ERR_HIP;
      L->ev_recorded[i] = false;
    }
    L->profiling = true;
  } else {
    L->profiling = false;
    for (int i = 0; i < LYNX_PROFILE_SLOTS; ++i) {
      (void)hipEventDestroy(L->ev_begin[i]);
      (void)hipEventDestroy(L->ev_end[i]);
      L->ev_recorded[i] = false;
    }
  }
  return LYNX_OK;
}

lynx_status lynx_layer_profile_ms(lynx_layer_t L, float* ms_out) {
  if (L == nullptr || ms_out == nullptr) return LYNX_ERR_INVALID_ARG;
  if (!L->profiling) return LYNX_ERR_STATE;
  for (int i = 0; i < LYNX_PROFILE_SLOTS; ++i) {
    ms_out[i] = -1.0f;
    if (!L->ev_recorded[i]) continue;
    if (hipEventSynchronize(L->ev_end[i]) != hipSuccess ||
        hipEventElapsedTime(&ms_out[i], L->ev_begin[i], L->ev_end[i]) != hipSuccess)
      return LYNX_ERR_HIP;
    L->ev_recorded[i] = false;
  }
  return LYNX_OK;
}

const char* lynx_profile_slot_name(int slot) {
  return (slot >= 1 && slot < kNumSlots) ? kSlotNames[slot] : "";
}

lynx_status lynx_policy_layer_problem(const lynx_layer_config* cfg, lynx_policy_problem* problem_out,
                                      uint32_t* parents_out, double* bytes_out) {
  if (cfg == nullptr || problem_out == nullptr || parents_out == nullptr || bytes_out == nullptr)
    return LYNX_ERR_INVALID_ARG;
  Dims D;
  if (!make_dims(cfg, &D)) return LYNX_ERR_SHAPE;
  for (int i = 1; i <= kNumOps; ++i) {
    uint32_t m = 0;
    for (int k = 0; k < 3 && kParents[i][k] >= 0; ++k) m |= 1u << kParents[i][k];
    parents_out[i - 1] = m;
    bytes_out[i - 1] = static_cast<double>(act_bytes(D, i));
  }
  problem_out->n_ops = kNumOps;
  problem_out->parents = parents_out;
  problem_out->bytes = bytes_out;
  problem_out->needed_mask = kBackwardNeeds;
  problem_out->comm_mask = 0;
  return LYNX_OK;
}

const char* lynx_status_string(lynx_status s) {
  switch (s) {
    case LYNX_OK: return "ok";
    case LYNX_ERR_INVALID_ARG: return "invalid argument";
    case LYNX_ERR_SHAPE: return "unsupported shape or configuration";
    case LYNX_ERR_STATE: return "call order violated";
    case LYNX_ERR_DEPENDENCY: return "recompute segment has an absent input";
    case LYNX_ERR_OOM: return "workspace too small";
    case LYNX_ERR_HIP: return "HIP call failed";
  }
  return "unknown status";
}

}  // extern "C"
