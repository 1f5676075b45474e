// Host side of the dense-tower C ABI (include/ctr_mlp.h): memory layout, the sequence of library
// bf16 GEMMs (hipBLASLt with a kernel chosen per product, rocBLAS as the fallback) and hand-written
// kernels of one training step, the dense optimizer and its merge.
#include "../../include/ctr_mlp.h"
#include "../../include/ctr_sparse.h"

#include <hipblaslt/hipblaslt.h>
#include <hipblaslt/hipblaslt-ext.hpp>
#include <rocblas/rocblas.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <new>
#include <vector>

#include "common.h"
#include "mlp_kernels.h"

using namespace ctr;

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
// Scratch a split-K product kernel may ask for: room for four partial copies of the largest weight
// gradient (products with a small result and a long contraction are split along the batch).
size_t lt_ws_bytes(const ctr_mlp_config* c) {
  size_t mx = 0;
  for (u32 l = 0; l < c->n_hidden; ++l)
    mx = std::max(mx, (size_t)(l == 0 ? c->in_dim : c->hidden[l - 1]) * c->hidden[l] * sizeof(float));
  return std::min<size_t>(std::max<size_t>(align256(4 * mx), (size_t)32 << 20), (size_t)512 << 20);
}
inline u32 blocks_for(u64 threads) { return (u32)((threads + BLOCK - 1) / BLOCK); }

bool mlp_config_ok(const ctr_mlp_config* c) {
  if (!c) return false;
  if (c->in_dim == 0 || c->in_dim % 8 != 0) return false;
  if (c->n_hidden == 0 || c->n_hidden > CTR_MLP_MAX_HIDDEN) return false;
  for (u32 i = 0; i < c->n_hidden; ++i)
    if (c->hidden[i] == 0 || c->hidden[i] % 8 != 0 || c->hidden[i] > 65536) return false;
  if (c->n_replicas == 0 || c->n_replicas > 31) return false;
  if (c->kstep > 1) return false;
  if (!c->kstep && c->n_replicas != 1) return false;
  if (!(c->lr > 0.0f) || !(c->beta1 >= 0.0f && c->beta1 < 1.0f) || !(c->beta2 >= 0.0f && c->beta2 < 1.0f) ||
      !(c->eps > 0.0f))
    return false;
  return true;
}

void make_layout(const ctr_mlp_config* c, MlpLayout* L) {
  L->n_layers = c->n_hidden + 1;
  u64 off = 0;
  for (u32 l = 0; l < L->n_layers; ++l) {
    L->in[l] = l == 0 ? c->in_dim : c->hidden[l - 1];
    L->out[l] = l < c->n_hidden ? c->hidden[l] : 1;
    L->w_off[l] = off;
    off += (u64)L->in[l] * L->out[l] + L->out[l];
  }
  L->n_params = off;
}

struct MemLayout {
  u64 stride;  // elements between replicas (n_params rounded up to 128)
  size_t off_params, off_m, off_v, off_pb, off_vhat, total;
};

void mem_layout(const ctr_mlp_config* c, const MlpLayout& L, MemLayout* M) {
  M->stride = (L.n_params + 127) & ~(u64)127;
  const size_t W = c->n_replicas;
  size_t o = 0;
  M->off_params = o; o += align256(M->stride * W * sizeof(float));
  M->off_m = o; o += align256(M->stride * W * sizeof(float));
  M->off_v = o; o += align256(M->stride * W * sizeof(float));
  M->off_pb = o; o += align256(M->stride * W * sizeof(bf16_t));
  M->off_vhat = o;
  if (c->kstep) o += align256(M->stride * sizeof(float));
  M->total = o;
}

struct WsLayout {
  u32 max_h;
  size_t off_h0, off_act[CTR_MLP_MAX_HIDDEN], off_z, off_da, off_dz[2], off_logits, off_dlogit, off_lterm, off_grads,
      off_partial, off_lt_ws, lt_ws, total;
};

void ws_layout(const ctr_mlp_config* c, const MlpLayout& L, u32 B, WsLayout* S) {
  u32 mh = 8;
  for (u32 i = 0; i < c->n_hidden; ++i) mh = std::max(mh, c->hidden[i]);
  S->max_h = mh;
  size_t o = 0;
  S->off_h0 = o; o += align256((size_t)B * c->in_dim * sizeof(bf16_t));
  for (u32 i = 0; i < c->n_hidden; ++i) {
    S->off_act[i] = o;
    o += align256((size_t)B * c->hidden[i] * sizeof(bf16_t));
  }
  S->off_z = o; o += align256((size_t)B * mh * sizeof(float));
  S->off_da = o; o += align256((size_t)B * mh * sizeof(float));
  S->off_dz[0] = o; o += align256((size_t)B * mh * sizeof(bf16_t));
  S->off_dz[1] = o; o += align256((size_t)B * mh * sizeof(bf16_t));
  S->off_logits = o; o += align256((size_t)B * sizeof(float));
  S->off_dlogit = o; o += align256((size_t)B * sizeof(float));
  S->off_lterm = o; o += align256((size_t)B * sizeof(double));
  S->off_grads = o; o += align256((size_t)L.n_params * sizeof(float));
  S->off_partial = o; o += align256((size_t)COLSUM_SLICES * mh * sizeof(float));
  S->off_lt_ws = o; S->lt_ws = lt_ws_bytes(c); o += S->lt_ws;
  S->total = o;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? CTR_OK : CTR_E_DEVICE; }

}  // namespace

// The three products of a hidden layer.  Row-major matrices are handed to the column-major
// library as the column-major matrices of their transposes ((XY)^T = Y^T X^T):
//   OP_FWD  Z[B x o]  = H[B x i] W[i x o]      -> gemm(N, N, m = o, n = B, k = i)
//   OP_DW   dW[i x o] = H^T[i x B] dZ[B x o]   -> gemm(N, T, m = o, n = i, k = B)
//   OP_DH   dH[B x i] = dZ[B x o] W^T[o x i]   -> gemm(T, N, m = i, n = B, k = o)
//   OP_DH16 the first layer's OP_DH with the result rounded to bf16 on the way out (the gradient of a
//           bf16 input handed back in the input's precision); planned for layer 0 only
enum { OP_FWD = 0, OP_DW = 1, OP_DH = 2, OP_DH16 = 3, N_OPS = 4 };

struct LtPlan {
  bool ready = false;  // descriptors exist and an algorithm was found
  bool tuned = false;  // the algorithm is the winner of ctr_mlp_tune, not the library's first guess
  hipblasLtMatmulDesc_t desc = nullptr;
  hipblasLtMatrixLayout_t la = nullptr, lb = nullptr, lc = nullptr;
  hipblasLtMatmulAlgo_t algo;
  size_t ws = 0;
  int m = 0, n = 0, k = 0;
};

struct ctr_mlp {
  ctr_mlp_config cfg;
  MlpLayout L;
  MemLayout M;
  char* mem;
  float *params, *m, *v, *vhat;
  bf16_t* pb;
  rocblas_handle blas;
  hipblasLtHandle_t lt;
  u32 plan_batch;  // batch size the plans were made for (0: none)
  LtPlan plans[CTR_MLP_MAX_HIDDEN][N_OPS];
  u32 pend_mask;  // replicas whose last step was a merge step not merged yet
};

namespace {

struct GemmShape {
  hipblasOperation_t opa, opb;
  int m, n, k, lda, ldb, ldc;
};

GemmShape shape_of(const MlpLayout& L, u32 l, int op, u32 B) {
  const int i = (int)L.in[l], o = (int)L.out[l], b = (int)B;
  switch (op) {
    case OP_FWD: return {HIPBLAS_OP_N, HIPBLAS_OP_N, o, b, i, o, i, o};
    case OP_DW: return {HIPBLAS_OP_N, HIPBLAS_OP_T, o, i, b, o, i, o};
    default: return {HIPBLAS_OP_T, HIPBLAS_OP_N, i, b, o, o, o, i};
  }
}

void destroy_plan(LtPlan* p) {
  if (p->desc) (void)hipblasLtMatmulDescDestroy(p->desc);
  if (p->la) (void)hipblasLtMatrixLayoutDestroy(p->la);
  if (p->lb) (void)hipblasLtMatrixLayoutDestroy(p->lb);
  if (p->lc) (void)hipblasLtMatrixLayoutDestroy(p->lc);
  *p = LtPlan();
}

void destroy_plans(ctr_mlp* t) {
  for (u32 l = 0; l < CTR_MLP_MAX_HIDDEN; ++l)
    for (int op = 0; op < N_OPS; ++op) destroy_plan(&t->plans[l][op]);
  t->plan_batch = 0;
}

// Descriptors of one product and the library's own first choice of kernel for it.
bool make_plan(ctr_mlp* t, u32 l, int op, u32 B, LtPlan* p) {
  const GemmShape g = shape_of(t->L, l, op, B);
  const bool ok = hipblasLtMatmulDescCreate(&p->desc, HIPBLAS_COMPUTE_32F, HIP_R_32F) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatmulDescSetAttribute(p->desc, HIPBLASLT_MATMUL_DESC_TRANSA, &g.opa, sizeof(g.opa)) ==
                      HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatmulDescSetAttribute(p->desc, HIPBLASLT_MATMUL_DESC_TRANSB, &g.opb, sizeof(g.opb)) ==
                      HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&p->la, HIP_R_16BF, g.opa == HIPBLAS_OP_N ? g.m : g.k,
                                              g.opa == HIPBLAS_OP_N ? g.k : g.m, g.lda) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&p->lb, HIP_R_16BF, g.opb == HIPBLAS_OP_N ? g.k : g.n,
                                              g.opb == HIPBLAS_OP_N ? g.n : g.k, g.ldb) == HIPBLAS_STATUS_SUCCESS &&
                  hipblasLtMatrixLayoutCreate(&p->lc, op == OP_DH16 ? HIP_R_16BF : HIP_R_32F, g.m, g.n, g.ldc) ==
                      HIPBLAS_STATUS_SUCCESS;
  if (!ok) return false;
  p->m = g.m; p->n = g.n; p->k = g.k;
  hipblasLtMatmulPreference_t pref = nullptr;
  if (hipblasLtMatmulPreferenceCreate(&pref) != HIPBLAS_STATUS_SUCCESS) return false;
  const uint64_t max_ws = lt_ws_bytes(&t->cfg);
  hipblasLtMatmulHeuristicResult_t res[4];
  int n_res = 0;
  bool found = hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &max_ws,
                                                      sizeof(max_ws)) == HIPBLAS_STATUS_SUCCESS &&
               hipblasLtMatmulAlgoGetHeuristic(t->lt, p->desc, p->la, p->lb, p->lc, p->lc, pref, 4, res, &n_res) ==
                   HIPBLAS_STATUS_SUCCESS;
  (void)hipblasLtMatmulPreferenceDestroy(pref);
  if (!found) return false;
  for (int r = 0; r < n_res; ++r) {
    if (res[r].state == HIPBLAS_STATUS_SUCCESS && res[r].workspaceSize <= max_ws) {
      p->algo = res[r].algo;
      p->ws = res[r].workspaceSize;
      p->ready = true;
      return true;
    }
  }
  return false;
}

// Plans are made for one batch size and kept until a call comes with another.
void ensure_plans(ctr_mlp* t, u32 B) {
  if (t->plan_batch == B || !t->lt) return;
  destroy_plans(t);
  for (u32 l = 0; l + 1 < t->L.n_layers; ++l)
    for (int op = 0; op < N_OPS; ++op)
      if ((op == OP_DH16 && l != 0) || !make_plan(t, l, op, B, &t->plans[l][op])) destroy_plan(&t->plans[l][op]);
  t->plan_batch = B;
}

// rocBLAS's default kernel for a product (bf16 operands, fp32 accumulation; the result fp32, or
// bf16 for OP_DH16).
bool rocblas_product(ctr_mlp* t, u32 l, int op, u32 B, const void* a, const void* b, void* c) {
  const float alpha = 1.0f, beta = 0.0f;
  const GemmShape g = shape_of(t->L, l, op, B);
  const rocblas_datatype ct = op == OP_DH16 ? rocblas_datatype_bf16_r : rocblas_datatype_f32_r;
  return rocblas_gemm_ex(t->blas, g.opa == HIPBLAS_OP_N ? rocblas_operation_none : rocblas_operation_transpose,
                         g.opb == HIPBLAS_OP_N ? rocblas_operation_none : rocblas_operation_transpose, g.m, g.n, g.k,
                         &alpha, a, rocblas_datatype_bf16_r, g.lda, b, rocblas_datatype_bf16_r, g.ldb, &beta, c, ct,
                         g.ldc, c, ct, g.ldc, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0) ==
         rocblas_status_success;
}

// One product on the matrix cores: the planned hipBLASLt kernel, else rocBLAS's default.
// c: fp32, except bf16 for OP_DH16.
bool product(ctr_mlp* t, u32 l, int op, u32 B, const void* a, const void* b, void* c, char* ws, const WsLayout& S,
             hipStream_t st) {
  const float alpha = 1.0f, beta = 0.0f;
  const LtPlan& p = t->plans[l][op];
  if (t->plan_batch == B && p.ready)
    return hipblasLtMatmul(t->lt, p.desc, &alpha, a, p.la, b, p.lb, &beta, c, p.lc, c, p.lc, &p.algo,
                           ws + S.off_lt_ws, p.ws, st) == HIPBLAS_STATUS_SUCCESS;
  return rocblas_product(t, l, op, B, a, b, c);
}

// ---------------------------------------------------------------- kernel search (ctr_mlp_tune)

size_t tune_result_bytes(const MlpLayout& L, u32 B) {
  size_t mx = 0;
  for (u32 l = 0; l + 1 < L.n_layers; ++l) {
    mx = std::max(mx, (size_t)B * L.out[l]);        // forward
    mx = std::max(mx, (size_t)L.in[l] * L.out[l]);  // weight gradient
    mx = std::max(mx, (size_t)B * L.in[l]);         // input gradient
  }
  return align256(mx * sizeof(float));
}

struct Tuner {
  ctr_mlp* t;
  hipStream_t st;
  char* ws;
  const WsLayout& S;
  u32* d_words;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok = false;

  Tuner(ctr_mlp* t_, hipStream_t st_, char* ws_, const WsLayout& S_, u32* d_words_)
      : t(t_), st(st_), ws(ws_), S(S_), d_words(d_words_) {
    if (hipEventCreate(&e0) != hipSuccess) return;
    if (hipEventCreate(&e1) != hipSuccess) return;
    ok = true;
  }
  ~Tuner() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }

  // Milliseconds of one run of `algo` into `out`, or a negative value if the library refuses it.
  float run(const LtPlan& p, const hipblasLtMatmulAlgo_t& algo, size_t wsz, const void* a, const void* b, void* out) {
    const float alpha = 1.0f, beta = 0.0f;
    if (hipEventRecord(e0, st) != hipSuccess) return -1.0f;
    const hipblasStatus_t rc = hipblasLtMatmul(t->lt, p.desc, &alpha, a, p.la, b, p.lb, &beta, out, p.lc, out, p.lc,
                                               &algo, ws + S.off_lt_ws, wsz, st);
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) return -1.0f;
    if (rc != HIPBLAS_STATUS_SUCCESS) return -1.0f;
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) return -1.0f;
    return ms;
  }

  bool read_words(u32 h[4]) {
    return hipMemcpyAsync(h, d_words, 4 * sizeof(u32), hipMemcpyDeviceToHost, st) == hipSuccess &&
           hipStreamSynchronize(st) == hipSuccess;
  }

  // The candidate agrees with the reference (accumulation order aside) and repeats bit for bit.
  // fp32 results: to 1e-3 of the largest element.  bf16 results (n even): two correct kernels may
  // round an element to neighbouring bf16 values, one unit in the last place of the largest
  // element (2^-7 of it) at most.
  bool valid(const LtPlan& p, const hipblasLtMatmulAlgo_t& algo, size_t wsz, const void* a, const void* b,
             const void* ref, void* cand, u64 n, bool out_bf16) {
    u32 h1[4], h2[4];
    for (int rep = 0; rep < 2; ++rep) {
      if (hipMemsetAsync(d_words, 0, 4 * sizeof(u32), st) != hipSuccess) return false;
      if (run(p, algo, wsz, a, b, cand) < 0.0f) return false;
      if (out_bf16) {
        hipLaunchKernelGGL(k_max_diff_bf16, dim3(2048), dim3(BLOCK), 0, st, (const bf16_t*)ref, (const bf16_t*)cand, n,
                           d_words);
        hipLaunchKernelGGL(k_hash_bits, dim3(2048), dim3(BLOCK), 0, st, (const float*)cand, n / 2,
                           (unsigned long long*)(d_words + 2));
      } else {
        hipLaunchKernelGGL(k_max_diff, dim3(2048), dim3(BLOCK), 0, st, (const float*)ref, (const float*)cand, n,
                           d_words);
        hipLaunchKernelGGL(k_hash_bits, dim3(2048), dim3(BLOCK), 0, st, (const float*)cand, n,
                           (unsigned long long*)(d_words + 2));
      }
      if (!read_words(rep ? h2 : h1)) return false;
    }
    float md, ma;
    memcpy(&md, &h1[0], 4);
    memcpy(&ma, &h1[1], 4);
    return md <= (out_bf16 ? 0.0078125f : 1e-3f) * ma && h1[2] == h2[2] && h1[3] == h2[3];
  }

  // Replaces the plan's kernel by the fastest applicable one that passes valid().  A product for
  // which nothing better is found keeps the library's choice.  Returns false on a device error only.
  bool tune_one(u32 l, int op, u32 B, float* ref, float* cand) {
    if (op == OP_DH16 && l != 0) return true;  // exists for the first layer only
    LtPlan& p = t->plans[l][op];
    if (!p.ready) {
      if (getenv("CTR_MLP_TUNE_LOG")) fprintf(stderr, "ctr_mlp_tune: layer %u product %d: no plan (rocBLAS runs it)\n", l, op);
      return true;
    }
    const MlpLayout& L = t->L;
    bf16_t* act_in = l == 0 ? (bf16_t*)(ws + S.off_h0) : (bf16_t*)(ws + S.off_act[l - 1]);  // B x in_l
    bf16_t* dzb = (bf16_t*)(ws + S.off_dz[0]);                                              // B x out_l
    const bf16_t* w = t->pb + L.w_off[l];
    const void* a = op == OP_DW ? (const void*)dzb : (const void*)w;
    const void* b = (op == OP_DH || op == OP_DH16) ? (const void*)dzb : (const void*)act_in;
    const u64 n = (u64)p.m * p.n;
    hipLaunchKernelGGL(k_fill_pattern_bf16, dim3(2048), dim3(BLOCK), 0, st, act_in, (u64)B * L.in[l], 0x1234u + l);
    hipLaunchKernelGGL(k_fill_pattern_bf16, dim3(2048), dim3(BLOCK), 0, st, dzb, (u64)B * L.out[l], 0x9876u + l);
    // reference: rocBLAS's own kernel for the same product
    if (!rocblas_product(t, l, op, B, a, b, ref)) return true;  // nothing to compare against: keep the plan as it is
    std::vector<hipblasLtMatmulHeuristicResult_t> all;
    const GemmShape g = shape_of(L, l, op, B);
    const hipDataType out_t = op == OP_DH16 ? HIP_R_16BF : HIP_R_32F;
    if (hipblaslt_ext::getAllAlgos(t->lt, hipblaslt_ext::GemmType::HIPBLASLT_GEMM, g.opa, g.opb, HIP_R_16BF, HIP_R_16BF,
                                   out_t, out_t, HIPBLAS_COMPUTE_32F, all) != HIPBLAS_STATUS_SUCCESS)
      return true;
    struct Timed { float ms; size_t idx, wsz; };
    std::vector<Timed> timed;
    size_t n_big = 0, n_sup = 0;
    const float alpha = 1.0f, beta = 0.0f;
    float best = run(p, p.algo, p.ws, a, b, cand);  // the current choice; the first run warms up
    best = run(p, p.algo, p.ws, a, b, cand);
    if (best >= 0.0f) best = std::min(best, run(p, p.algo, p.ws, a, b, cand));
    if (best < 0.0f) {
      if (getenv("CTR_MLP_TUNE_LOG")) fprintf(stderr, "ctr_mlp_tune: layer %u product %d: the planned kernel does not run\n", l, op);
      return hipGetLastError() == hipSuccess;
    }
    const float current = best;
    for (size_t i = 0; i < all.size(); ++i) {
      size_t wsz = 0;
      if (hipblaslt_ext::matmulIsAlgoSupported(t->lt, p.desc, &alpha, p.la, p.lb, &beta, p.lc, p.lc, all[i].algo, wsz) !=
          HIPBLAS_STATUS_SUCCESS)
        continue;
      if (wsz > S.lt_ws) { ++n_big; continue; }
      ++n_sup;
      if (run(p, all[i].algo, wsz, a, b, cand) < 0.0f) continue;  // the first run of a kernel pays for loading it
      float ms = run(p, all[i].algo, wsz, a, b, cand);
      if (ms < 0.0f) continue;
      if (ms < 1.1f * best) {  // a contender: one more look
        const float ms2 = run(p, all[i].algo, wsz, a, b, cand);
        if (ms2 >= 0.0f) ms = std::min(ms, ms2);
      }
      best = std::min(best, ms);
      timed.push_back({ms, i, wsz});
    }
    std::sort(timed.begin(), timed.end(), [](const Timed& x, const Timed& y) { return x.ms < y.ms; });
    const bool log = getenv("CTR_MLP_TUNE_LOG") != nullptr;
    if (log)
      fprintf(stderr, "ctr_mlp_tune: layer %u product %d (m %d n %d k %d): library's choice %.3f ms (index %d), %zu listed, %zu applicable, %zu need more scratch, %zu ran, fastest %.3f ms\n",
              l, op, p.m, p.n, p.k, current, hipblaslt_ext::getIndexFromAlgo(p.algo), all.size(), n_sup, n_big, timed.size(), timed.empty() ? -1.0f : timed[0].ms);
    if (log)
      for (size_t r = 0; r < std::min<size_t>(timed.size(), 4); ++r)
        fprintf(stderr, "ctr_mlp_tune:   #%zu %.3f ms ws %zu index %d %s\n", r, timed[r].ms, timed[r].wsz,
                hipblaslt_ext::getIndexFromAlgo(all[timed[r].idx].algo),
                hipblaslt_ext::getKernelNameFromAlgo(t->lt, all[timed[r].idx].algo).substr(0, 110).c_str());
    for (const Timed& c : timed) {
      if (c.ms >= 0.97f * current) break;  // not better than what the library chose by itself
      const bool good = valid(p, all[c.idx].algo, c.wsz, a, b, ref, cand, n, op == OP_DH16);
      if (log) fprintf(stderr, "ctr_mlp_tune:   candidate %zu at %.3f ms: %s\n", c.idx, c.ms, good ? "taken" : "rejected");
      if (good) {
        p.algo = all[c.idx].algo;
        p.ws = c.wsz;
        p.tuned = true;
        break;
      }
    }
    return hipGetLastError() == hipSuccess;
  }
};

// Forward through the hidden layers and the output layer; activations stay in the workspace.
// The input is either fp32 (rounded to bf16 into the workspace) or already bf16 (used in place).
bool forward(ctr_mlp* t, u32 replica, const float* d_pooled, const bf16_t* d_pooled_bf16, u32 B, char* ws,
             const WsLayout& S, float* logits, hipStream_t st) {
  const MlpLayout& L = t->L;
  const float* P = t->params + (u64)replica * t->M.stride;
  const bf16_t* PB = t->pb + (u64)replica * t->M.stride;
  const bf16_t* h = d_pooled_bf16;
  float* z = (float*)(ws + S.off_z);
  if (!h) {
    const u64 n0 = (u64)B * L.in[0];
    hipLaunchKernelGGL(k_cast_bf16, dim3(blocks_for(n0 / 4)), dim3(BLOCK), 0, st, d_pooled, (bf16_t*)(ws + S.off_h0), n0);
    h = (const bf16_t*)(ws + S.off_h0);
  }
  for (u32 l = 0; l + 1 < L.n_layers; ++l) {
    const int i = (int)L.in[l], o = (int)L.out[l];
    if (!product(t, l, OP_FWD, B, PB + L.w_off[l], h, z, ws, S, st)) return false;
    bf16_t* a = (bf16_t*)(ws + S.off_act[l]);
    const u64 n = (u64)B * o;
    hipLaunchKernelGGL(k_bias_relu_bf16, dim3(blocks_for(n / 4)), dim3(BLOCK), 0, st, z,
                       P + L.w_off[l] + (u64)i * o, (u32)o, n, a);
    h = a;
  }
  const u32 lo = L.n_layers - 1;
  hipLaunchKernelGGL(k_out_forward, dim3(blocks_for((u64)B * WAVE)), dim3(BLOCK), 0, st, h, PB + L.w_off[lo],
                     P + L.w_off[lo] + L.in[lo], B, L.in[lo], logits);
  return true;
}

}  // namespace

extern "C" {

size_t ctr_mlp_n_params(const ctr_mlp_config* cfg) {
  if (!mlp_config_ok(cfg)) return 0;
  MlpLayout L;
  make_layout(cfg, &L);
  return (size_t)L.n_params;
}

size_t ctr_mlp_bytes(const ctr_mlp_config* cfg) {
  if (!mlp_config_ok(cfg)) return 0;
  MlpLayout L;
  MemLayout M;
  make_layout(cfg, &L);
  mem_layout(cfg, L, &M);
  return M.total;
}

size_t ctr_mlp_workspace_bytes(const ctr_mlp_config* cfg, uint32_t batch) {
  if (!mlp_config_ok(cfg) || batch == 0 || batch % 8 != 0 || batch > CTR_MLP_MAX_BATCH) return 0;
  MlpLayout L;
  WsLayout S;
  make_layout(cfg, &L);
  ws_layout(cfg, L, batch, &S);
  return S.total;
}

int ctr_mlp_create(const ctr_mlp_config* cfg, void* d_mem, size_t bytes, void* hip_stream, ctr_mlp** out) {
  if (!cfg || !d_mem || !out) return CTR_E_INVAL;
  if (!mlp_config_ok(cfg)) return CTR_E_INVAL;
  if (((uintptr_t)d_mem & 255) != 0) return CTR_E_INVAL;
  ctr_mlp* t = new (std::nothrow) ctr_mlp();
  if (!t) return CTR_E_NOMEM;
  t->cfg = *cfg;
  make_layout(cfg, &t->L);
  mem_layout(cfg, t->L, &t->M);
  if (bytes < t->M.total) {
    delete t;
    return CTR_E_NOMEM;
  }
  t->mem = (char*)d_mem;
  t->params = (float*)(t->mem + t->M.off_params);
  t->m = (float*)(t->mem + t->M.off_m);
  t->v = (float*)(t->mem + t->M.off_v);
  t->pb = (bf16_t*)(t->mem + t->M.off_pb);
  t->vhat = cfg->kstep ? (float*)(t->mem + t->M.off_vhat) : nullptr;
  t->pend_mask = 0;
  if (rocblas_create_handle(&t->blas) != rocblas_status_success) {
    delete t;
    return CTR_E_DEVICE;
  }
  // CTR_MLP_NO_HIPBLASLT in the environment (or a hipBLASLt that cannot start) sends the products through rocBLAS
  if (getenv("CTR_MLP_NO_HIPBLASLT") != nullptr || hipblasLtCreate(&t->lt) != HIPBLAS_STATUS_SUCCESS) t->lt = nullptr;
  t->plan_batch = 0;
  // fixed summation order: no atomics in the products
  (void)rocblas_set_atomics_mode(t->blas, rocblas_atomics_not_allowed);
  (void)rocblas_set_pointer_mode(t->blas, rocblas_pointer_mode_host);
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(k_mlp_init, dim3(blocks_for(t->L.n_params)), dim3(BLOCK), 0, st, t->L,
                     cfg->init_seed * 0x9E3779B97F4A7C15ull, cfg->eps, cfg->n_replicas, t->M.stride, t->params, t->m,
                     t->v, t->vhat, t->pb);
  if (launch_status() != CTR_OK) {
    (void)rocblas_destroy_handle(t->blas);
    if (t->lt) (void)hipblasLtDestroy(t->lt);
    delete t;
    return CTR_E_DEVICE;
  }
  *out = t;
  return CTR_OK;
}

int ctr_mlp_destroy(ctr_mlp* t) {
  if (!t) return CTR_E_INVAL;
  destroy_plans(t);
  (void)rocblas_destroy_handle(t->blas);
  if (t->lt) (void)hipblasLtDestroy(t->lt);
  delete t;
  return CTR_OK;
}

static int mlp_forward_impl(ctr_mlp* t, uint32_t replica, const float* d_pooled, const bf16_t* d_pooled_bf16,
                            uint32_t batch, float* d_logits, void* d_workspace, size_t workspace_bytes,
                            void* hip_stream) {
  if (!t || (!d_pooled && !d_pooled_bf16) || !d_logits || !d_workspace) return CTR_E_INVAL;
  if (replica >= t->cfg.n_replicas || batch == 0 || batch % 8 != 0 || batch > CTR_MLP_MAX_BATCH) return CTR_E_INVAL;
  if (((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WsLayout S;
  ws_layout(&t->cfg, t->L, batch, &S);
  if (workspace_bytes < S.total) return CTR_E_NOMEM;
  hipStream_t st = (hipStream_t)hip_stream;
  if (rocblas_set_stream(t->blas, st) != rocblas_status_success) return CTR_E_DEVICE;
  ensure_plans(t, batch);
  if (!forward(t, replica, d_pooled, d_pooled_bf16, batch, (char*)d_workspace, S, d_logits, st)) return CTR_E_DEVICE;
  return launch_status();
}

// The gradient of the pooled input goes to d_grad_pooled (fp32) or to d_grad_pooled_bf16: exactly one is given.
static int mlp_step_impl(ctr_mlp* t, uint32_t replica, const float* d_pooled, const bf16_t* d_pooled_bf16,
                         const float* d_labels, uint32_t batch, float* d_grad_pooled, bf16_t* d_grad_pooled_bf16,
                         float* d_loss, void* d_workspace, size_t workspace_bytes, uint32_t mode, void* hip_stream) {
  if (!t || (!d_pooled && !d_pooled_bf16) || !d_labels || (!d_grad_pooled == !d_grad_pooled_bf16) || !d_loss ||
      !d_workspace)
    return CTR_E_INVAL;
  if (replica >= t->cfg.n_replicas || batch == 0 || batch % 8 != 0 || batch > CTR_MLP_MAX_BATCH) return CTR_E_INVAL;
  if (mode != CTR_STEP_LOCAL && mode != CTR_STEP_MERGE_PENDING) return CTR_E_INVAL;
  if (!t->cfg.kstep && mode != CTR_STEP_LOCAL) return CTR_E_INVAL;
  if (((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WsLayout S;
  ws_layout(&t->cfg, t->L, batch, &S);
  if (workspace_bytes < S.total) return CTR_E_NOMEM;
  hipStream_t st = (hipStream_t)hip_stream;
  if (rocblas_set_stream(t->blas, st) != rocblas_status_success) return CTR_E_DEVICE;
  ensure_plans(t, batch);

  const MlpLayout& L = t->L;
  char* ws = (char*)d_workspace;
  const u32 B = batch;
  float* logits = (float*)(ws + S.off_logits);
  float* dlogit = (float*)(ws + S.off_dlogit);
  float* grads = (float*)(ws + S.off_grads);
  float* partial = (float*)(ws + S.off_partial);
  float* da = (float*)(ws + S.off_da);
  const bf16_t* PB = t->pb + (u64)replica * t->M.stride;

  double* lterm = (double*)(ws + S.off_lterm);
  const bf16_t* h0 = d_pooled_bf16 ? d_pooled_bf16 : (const bf16_t*)(ws + S.off_h0);
  if (!forward(t, replica, d_pooled, d_pooled_bf16, B, ws, S, logits, st)) return CTR_E_DEVICE;
  hipLaunchKernelGGL(k_bce, dim3(blocks_for(B)), dim3(BLOCK), 0, st, logits, d_labels, B, dlogit, lterm);
  hipLaunchKernelGGL(k_loss_mean, dim3(1), dim3(BLOCK), 0, st, lterm, B, d_loss);

  // output layer: weight and bias gradients, then back through the last ReLU
  const u32 lo = L.n_layers - 1;
  const u32 Hl = L.in[lo];
  const bf16_t* a_last = (const bf16_t*)(ws + S.off_act[lo - 1]);
  hipLaunchKernelGGL(k_colsum_partial, dim3((Hl + 31) / 32, COLSUM_SLICES), dim3(BLOCK), 0, st, a_last, dlogit, B, Hl,
                     partial);
  hipLaunchKernelGGL(k_colsum_final, dim3(blocks_for(Hl)), dim3(BLOCK), 0, st, partial, Hl, grads + L.w_off[lo]);
  hipLaunchKernelGGL(k_sum_f32, dim3(1), dim3(BLOCK), 0, st, dlogit, B, grads + L.w_off[lo] + Hl);
  bf16_t* dz = (bf16_t*)(ws + S.off_dz[0]);
  bf16_t* dz_next = (bf16_t*)(ws + S.off_dz[1]);
  {
    const u64 n = (u64)B * Hl;
    hipLaunchKernelGGL(k_out_backward_dz, dim3(blocks_for(n)), dim3(BLOCK), 0, st, a_last, dlogit, PB + L.w_off[lo],
                       Hl, n, dz);
  }
  // hidden layers, last to first
  for (int l = (int)lo - 1; l >= 0; --l) {
    const int i = (int)L.in[l], o = (int)L.out[l];
    const bf16_t* h_prev = l == 0 ? h0 : (const bf16_t*)(ws + S.off_act[l - 1]);
    if (!product(t, (u32)l, OP_DW, B, dz, h_prev, grads + L.w_off[l], ws, S, st)) return CTR_E_DEVICE;
    hipLaunchKernelGGL(k_colsum_partial, dim3((o + 31) / 32, COLSUM_SLICES), dim3(BLOCK), 0, st, dz, (const float*)nullptr,
                       B, (u32)o, partial);
    hipLaunchKernelGGL(k_colsum_final, dim3(blocks_for(o)), dim3(BLOCK), 0, st, partial, (u32)o,
                       grads + L.w_off[l] + (u64)i * o);
    // dH_prev[B x i] = dZ[B x o] W^T[o x i]; for the first layer this is the gradient of the pooled input
    if (l == 0 && d_grad_pooled_bf16) {
      if (!product(t, 0, OP_DH16, B, PB + L.w_off[0], dz, d_grad_pooled_bf16, ws, S, st)) return CTR_E_DEVICE;
    } else {
      float* dst = l == 0 ? d_grad_pooled : da;
      if (!product(t, (u32)l, OP_DH, B, PB + L.w_off[l], dz, dst, ws, S, st)) return CTR_E_DEVICE;
    }
    if (l > 0) {
      const u64 n = (u64)B * i;
      hipLaunchKernelGGL(k_relu_bwd_bf16, dim3(blocks_for(n / 4)), dim3(BLOCK), 0, st, da, h_prev, n, dz_next);
      std::swap(dz, dz_next);
    }
  }
  // dense optimizer
  const u32 amode = mode == CTR_STEP_MERGE_PENDING ? 2u : (t->cfg.kstep ? 1u : 0u);
  hipLaunchKernelGGL(k_dense_adam, dim3(blocks_for(L.n_params)), dim3(BLOCK), 0, st,
                     t->params + (u64)replica * t->M.stride, t->m + (u64)replica * t->M.stride,
                     t->v + (u64)replica * t->M.stride, t->vhat, grads, t->pb + (u64)replica * t->M.stride,
                     L.n_params, (double)t->cfg.beta1, (double)t->cfg.beta2, (double)t->cfg.lr, amode);
  if (mode == CTR_STEP_MERGE_PENDING) t->pend_mask |= 1u << replica;
  return launch_status();
}

int ctr_mlp_forward(ctr_mlp* t, uint32_t replica, const float* d_pooled, uint32_t batch, float* d_logits,
                    void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!d_pooled) return CTR_E_INVAL;
  return mlp_forward_impl(t, replica, d_pooled, nullptr, batch, d_logits, d_workspace, workspace_bytes, hip_stream);
}

int ctr_mlp_forward_bf16(ctr_mlp* t, uint32_t replica, const uint16_t* d_pooled_bf16, uint32_t batch,
                         float* d_logits, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!d_pooled_bf16) return CTR_E_INVAL;
  return mlp_forward_impl(t, replica, nullptr, d_pooled_bf16, batch, d_logits, d_workspace, workspace_bytes,
                          hip_stream);
}

int ctr_mlp_step(ctr_mlp* t, uint32_t replica, const float* d_pooled, const float* d_labels, uint32_t batch,
                 float* d_grad_pooled, float* d_loss, void* d_workspace, size_t workspace_bytes, uint32_t mode,
                 void* hip_stream) {
  if (!d_pooled) return CTR_E_INVAL;
  return mlp_step_impl(t, replica, d_pooled, nullptr, d_labels, batch, d_grad_pooled, nullptr, d_loss, d_workspace,
                       workspace_bytes, mode, hip_stream);
}

int ctr_mlp_step_bf16(ctr_mlp* t, uint32_t replica, const uint16_t* d_pooled_bf16, const float* d_labels,
                      uint32_t batch, float* d_grad_pooled, float* d_loss, void* d_workspace,
                      size_t workspace_bytes, uint32_t mode, void* hip_stream) {
  if (!d_pooled_bf16) return CTR_E_INVAL;
  return mlp_step_impl(t, replica, nullptr, d_pooled_bf16, d_labels, batch, d_grad_pooled, nullptr, d_loss,
                       d_workspace, workspace_bytes, mode, hip_stream);
}

int ctr_mlp_step_bf16_grad_bf16(ctr_mlp* t, uint32_t replica, const uint16_t* d_pooled_bf16, const float* d_labels,
                                uint32_t batch, uint16_t* d_grad_pooled_bf16, float* d_loss, void* d_workspace,
                                size_t workspace_bytes, uint32_t mode, void* hip_stream) {
  if (!d_pooled_bf16 || !d_grad_pooled_bf16) return CTR_E_INVAL;
  return mlp_step_impl(t, replica, nullptr, d_pooled_bf16, d_labels, batch, nullptr, d_grad_pooled_bf16, d_loss,
                       d_workspace, workspace_bytes, mode, hip_stream);
}

size_t ctr_mlp_tune_workspace_bytes(const ctr_mlp_config* cfg, uint32_t batch) {
  if (!mlp_config_ok(cfg) || batch == 0 || batch % 8 != 0 || batch > CTR_MLP_MAX_BATCH) return 0;
  MlpLayout L;
  WsLayout S;
  make_layout(cfg, &L);
  ws_layout(cfg, L, batch, &S);
  return S.total + 2 * tune_result_bytes(L, batch) + 256;
}

int ctr_mlp_tune(ctr_mlp* t, uint32_t batch, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!t || !d_workspace) return CTR_E_INVAL;
  if (batch == 0 || batch % 8 != 0 || batch > CTR_MLP_MAX_BATCH) return CTR_E_INVAL;
  if (((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WsLayout S;
  ws_layout(&t->cfg, t->L, batch, &S);
  const size_t res_bytes = tune_result_bytes(t->L, batch);
  if (workspace_bytes < S.total + 2 * res_bytes + 256) return CTR_E_NOMEM;
  if (!t->lt) return CTR_OK;  // no kernel to choose: the products run through rocBLAS
  hipStream_t st = (hipStream_t)hip_stream;
  if (rocblas_set_stream(t->blas, st) != rocblas_status_success) return CTR_E_DEVICE;
  ensure_plans(t, batch);
  char* ws = (char*)d_workspace;
  float* ref = (float*)(ws + S.total);
  float* cand = (float*)(ws + S.total + res_bytes);
  u32* d_words = (u32*)(ws + S.total + 2 * res_bytes);  // [0..1] max diff / max abs, [2..3] a 64-bit hash
  Tuner tu(t, st, ws, S, d_words);
  if (!tu.ok) return CTR_E_DEVICE;
  try {  // the candidate lists are host containers: no exception may cross the C boundary
    for (u32 l = 0; l + 1 < t->L.n_layers; ++l)
      for (int op = 0; op < N_OPS; ++op)
        if (!tu.tune_one(l, op, batch, ref, cand)) return CTR_E_DEVICE;
  } catch (const std::bad_alloc&) {
    return CTR_E_NOMEM;
  } catch (...) {
    return CTR_E_DEVICE;
  }
  return launch_status();
}

int ctr_mlp_kstep_merge(ctr_mlp* t, void* hip_stream) {
  if (!t || !t->cfg.kstep) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(k_dense_merge, dim3(blocks_for(t->L.n_params)), dim3(BLOCK), 0, st, t->params, t->m, t->v,
                     t->vhat, t->pb, t->L.n_params, t->M.stride, t->cfg.n_replicas, t->pend_mask,
                     (double)t->cfg.lr);
  t->pend_mask = 0;
  return launch_status();
}

int ctr_mlp_export(ctr_mlp* t, uint32_t replica, float* h_params, float* h_m, float* h_v, float* h_vhat,
                   void* hip_stream) {
  if (!t || replica >= t->cfg.n_replicas) return CTR_E_INVAL;
  if (h_vhat && !t->vhat) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t nb = (size_t)t->L.n_params * sizeof(float);
  const u64 off = (u64)replica * t->M.stride;
  bool ok = true;
  if (h_params) ok = ok && hipMemcpyAsync(h_params, t->params + off, nb, hipMemcpyDeviceToHost, st) == hipSuccess;
  if (h_m) ok = ok && hipMemcpyAsync(h_m, t->m + off, nb, hipMemcpyDeviceToHost, st) == hipSuccess;
  if (h_v) ok = ok && hipMemcpyAsync(h_v, t->v + off, nb, hipMemcpyDeviceToHost, st) == hipSuccess;
  if (h_vhat) ok = ok && hipMemcpyAsync(h_vhat, t->vhat, nb, hipMemcpyDeviceToHost, st) == hipSuccess;
  ok = ok && hipStreamSynchronize(st) == hipSuccess;
  return ok ? CTR_OK : CTR_E_DEVICE;
}

int ctr_mlp_import(ctr_mlp* t, uint32_t replica, const float* h_params, const float* h_m, const float* h_v,
                   const float* h_vhat, uint32_t pending, void* hip_stream) {
  if (!t || replica >= t->cfg.n_replicas) return CTR_E_INVAL;
  if (h_vhat && !t->vhat) return CTR_E_INVAL;
  if (pending > 1 || (pending && !t->cfg.kstep)) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t nb = (size_t)t->L.n_params * sizeof(float);
  const u64 off = (u64)replica * t->M.stride;
  bool ok = true;
  if (h_params) ok = ok && hipMemcpyAsync(t->params + off, h_params, nb, hipMemcpyHostToDevice, st) == hipSuccess;
  if (h_m) ok = ok && hipMemcpyAsync(t->m + off, h_m, nb, hipMemcpyHostToDevice, st) == hipSuccess;
  if (h_v) ok = ok && hipMemcpyAsync(t->v + off, h_v, nb, hipMemcpyHostToDevice, st) == hipSuccess;
  if (h_vhat) ok = ok && hipMemcpyAsync(t->vhat, h_vhat, nb, hipMemcpyHostToDevice, st) == hipSuccess;
  if (!ok) return CTR_E_DEVICE;
  if (h_params)
    hipLaunchKernelGGL(k_refresh_bf16, dim3(blocks_for(t->L.n_params)), dim3(BLOCK), 0, st, t->params + off,
                       t->pb + off, t->L.n_params);
  ok = hipStreamSynchronize(st) == hipSuccess;  // the host arrays may be pageable: they are free again on return
  t->pend_mask = pending ? (t->pend_mask | (1u << replica)) : (t->pend_mask & ~(1u << replica));
  return ok ? launch_status() : CTR_E_DEVICE;
}

}  // extern "C"
