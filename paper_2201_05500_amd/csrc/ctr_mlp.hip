// Host side of the dense-tower C ABI (include/ctr_mlp.h): memory layout, the sequence of hand-written
// kernels of one training step (the bf16 matrix products of gemm_kernels.h with their fused epilogues, the
// element-wise kernels of mlp_kernels.h), the dense optimizer and its merge.
#include "../../include/ctr_mlp.h"
#include "../../include/ctr_sparse.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"
#include "gemm_kernels.h"
#include "mlp_kernels.h"

using namespace ctr;

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
// Scratch for products whose contraction is split over several workgroups (gemm_kernels.h): room for
// four fp32 partial copies of the largest weight gradient, at least 32 MiB, at most 512 MiB.  A product
// that would need more is split less.
size_t gemm_scratch_bytes(const ctr_mlp_config* c) {
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
  size_t off_h0, off_act[CTR_MLP_MAX_HIDDEN], off_dz[2], off_logits, off_dlogit, off_lterm, off_grads, off_partial,
      off_gemm, gemm_bytes, total;
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
  S->off_dz[0] = o; o += align256((size_t)B * mh * sizeof(bf16_t));
  S->off_dz[1] = o; o += align256((size_t)B * mh * sizeof(bf16_t));
  S->off_logits = o; o += align256((size_t)B * sizeof(float));
  S->off_dlogit = o; o += align256((size_t)B * sizeof(float));
  S->off_lterm = o; o += align256((size_t)B * sizeof(double));
  S->off_grads = o; o += align256((size_t)L.n_params * sizeof(float));
  S->off_partial = o; o += align256((size_t)COLSUM_SLICES * mh * sizeof(float));
  S->off_gemm = o; S->gemm_bytes = gemm_scratch_bytes(c); o += S->gemm_bytes;
  S->total = o;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? CTR_OK : CTR_E_DEVICE; }

}  // namespace

struct ctr_mlp {
  ctr_mlp_config cfg;
  MlpLayout L;
  MemLayout M;
  char* mem;
  float *params, *m, *v, *vhat;
  bf16_t* pb;
  u32 pend_mask;  // replicas whose last step was a merge step not merged yet
};

namespace {

// The three products of a hidden layer with row-major matrices, as C[M x N] = A B of gemm_kernels.h
// (which operand is stored with the contraction index contiguous differs from product to product):
//   forward          act[B x o]  = bf16(relu(H[B x i] W[i x o] + bias))     A = H (k-contiguous), B = W (n-contiguous)
//   weight gradient  dW[i x o]   = H^T[i x B] dZ[B x o]                     A = H (m-contiguous), B = dZ (n-contiguous)
//   input gradient   dH[B x i]   = dZ[B x o] W^T[o x i]                     A = dZ (k-contiguous), B = W (k-contiguous)
// The input gradient of a hidden layer goes straight through the ReLU of the layer below (mask = that
// layer's activation) and is stored as bf16; the first layer's is the gradient of the pooled input,
// stored as fp32 or bf16.
bool product_forward(const MlpLayout& L, u32 l, u32 B, const bf16_t* h, const bf16_t* w, const float* bias,
                     bf16_t* act, char* ws, const WsLayout& S, hipStream_t st) {
  GemmArgs g{};
  g.A = h; g.lda = L.in[l];
  g.B = w; g.ldb = L.out[l];
  g.M = B; g.N = L.out[l]; g.K = L.in[l];
  g.C16 = act; g.ldc = L.out[l];
  g.bias = bias;
  g.epilogue = EPI_BIAS_RELU_BF16;
  return gemm_enqueue(true, false, g, (float*)(ws + S.off_gemm), S.gemm_bytes, st) == hipSuccess;
}

bool product_weight_grad(const MlpLayout& L, u32 l, u32 B, const bf16_t* h, const bf16_t* dz, float* dw, char* ws,
                         const WsLayout& S, hipStream_t st) {
  GemmArgs g{};
  g.A = h; g.lda = L.in[l];
  g.B = dz; g.ldb = L.out[l];
  g.M = L.in[l]; g.N = L.out[l]; g.K = B;
  g.C32 = dw; g.ldc = L.out[l];
  g.epilogue = EPI_F32;
  return gemm_enqueue(false, false, g, (float*)(ws + S.off_gemm), S.gemm_bytes, st) == hipSuccess;
}

// exactly one of out32 / out16 / (mask, out16): fp32, bf16, or bf16 gated by the sign of `mask`
bool product_input_grad(const MlpLayout& L, u32 l, u32 B, const bf16_t* dz, const bf16_t* w, float* out32,
                        bf16_t* out16, const bf16_t* mask, char* ws, const WsLayout& S, hipStream_t st) {
  GemmArgs g{};
  g.A = dz; g.lda = L.out[l];
  g.B = w; g.ldb = L.out[l];
  g.M = B; g.N = L.in[l]; g.K = L.out[l];
  g.C32 = out32; g.C16 = out16; g.ldc = L.in[l];
  g.mask = mask;
  g.epilogue = out32 ? EPI_F32 : (mask ? EPI_RELU_MASK_BF16 : EPI_BF16);
  return gemm_enqueue(true, true, g, (float*)(ws + S.off_gemm), S.gemm_bytes, st) == hipSuccess;
}

// Forward through the hidden layers and the output layer; activations stay in the workspace.
// The input is either fp32 (rounded to bf16 into the workspace) or already bf16 (used in place).
bool forward(ctr_mlp* t, u32 replica, const float* d_pooled, const bf16_t* d_pooled_bf16, u32 B, char* ws,
             const WsLayout& S, float* logits, hipStream_t st) {
  const MlpLayout& L = t->L;
  const float* P = t->params + (u64)replica * t->M.stride;
  const bf16_t* PB = t->pb + (u64)replica * t->M.stride;
  const bf16_t* h = d_pooled_bf16;
  if (!h) {
    const u64 n0 = (u64)B * L.in[0];
    hipLaunchKernelGGL(k_cast_bf16, dim3(blocks_for(n0 / 4)), dim3(BLOCK), 0, st, d_pooled, (bf16_t*)(ws + S.off_h0), n0);
    h = (const bf16_t*)(ws + S.off_h0);
  }
  for (u32 l = 0; l + 1 < L.n_layers; ++l) {
    bf16_t* a = (bf16_t*)(ws + S.off_act[l]);
    if (!product_forward(L, l, B, h, PB + L.w_off[l], P + L.w_off[l] + (u64)L.in[l] * L.out[l], a, ws, S, st)) return false;
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
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(k_mlp_init, dim3(blocks_for(t->L.n_params)), dim3(BLOCK), 0, st, t->L,
                     cfg->init_seed * 0x9E3779B97F4A7C15ull, cfg->eps, cfg->n_replicas, t->M.stride, t->params, t->m,
                     t->v, t->vhat, t->pb);
  if (launch_status() != CTR_OK) {
    delete t;
    return CTR_E_DEVICE;
  }
  *out = t;
  return CTR_OK;
}

int ctr_mlp_destroy(ctr_mlp* t) {
  if (!t) return CTR_E_INVAL;
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

  const MlpLayout& L = t->L;
  char* ws = (char*)d_workspace;
  const u32 B = batch;
  float* logits = (float*)(ws + S.off_logits);
  float* dlogit = (float*)(ws + S.off_dlogit);
  float* grads = (float*)(ws + S.off_grads);
  float* partial = (float*)(ws + S.off_partial);
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
    if (!product_weight_grad(L, (u32)l, B, h_prev, dz, grads + L.w_off[l], ws, S, st)) return CTR_E_DEVICE;
    hipLaunchKernelGGL(k_colsum_partial, dim3((o + 31) / 32, COLSUM_SLICES), dim3(BLOCK), 0, st, dz, (const float*)nullptr,
                       B, (u32)o, partial);
    hipLaunchKernelGGL(k_colsum_final, dim3(blocks_for(o)), dim3(BLOCK), 0, st, partial, (u32)o,
                       grads + L.w_off[l] + (u64)i * o);
    // dH_prev[B x i] = dZ[B x o] W^T[o x i]: for the first layer the gradient of the pooled input; for a hidden
    // layer gated by the ReLU below and rounded to bf16 on the way out (the next dZ)
    if (l == 0) {
      if (!product_input_grad(L, 0, B, dz, PB + L.w_off[0], d_grad_pooled, d_grad_pooled_bf16, nullptr, ws, S, st))
        return CTR_E_DEVICE;
    } else {
      if (!product_input_grad(L, (u32)l, B, dz, PB + L.w_off[l], nullptr, dz_next, h_prev, ws, S, st)) return CTR_E_DEVICE;
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

// The tower's matrix product on its own (testing and measurement): C32[M x N] = A B.
int ctr_mlp_gemm(int a_k_contiguous, int b_k_contiguous, const uint16_t* d_a, uint32_t lda, const uint16_t* d_b,
                 uint32_t ldb, uint32_t m, uint32_t n, uint32_t k, float* d_c, uint32_t ldc, void* d_scratch,
                 size_t scratch_bytes, void* hip_stream) {
  if (!d_a || !d_b || !d_c) return CTR_E_INVAL;
  if (m == 0 || n == 0 || k == 0 || ((m | n | k | lda | ldb | ldc) % 8u) != 0u) return CTR_E_INVAL;
  if (lda < (a_k_contiguous ? k : m) || ldb < (b_k_contiguous ? k : n) || ldc < n) return CTR_E_INVAL;
  if ((((uintptr_t)d_a | (uintptr_t)d_b | (uintptr_t)d_c | (uintptr_t)d_scratch) & 15) != 0) return CTR_E_INVAL;
  GemmArgs g{};
  g.A = d_a; g.lda = lda;
  g.B = d_b; g.ldb = ldb;
  g.M = m; g.N = n; g.K = k;
  g.C32 = d_c; g.ldc = ldc;
  g.epilogue = EPI_F32;
  const hipError_t rc = gemm_enqueue(a_k_contiguous != 0, b_k_contiguous != 0, g, (float*)d_scratch,
                                     d_scratch ? scratch_bytes : 0, (hipStream_t)hip_stream);
  return rc == hipSuccess ? CTR_OK : (rc == hipErrorInvalidValue ? CTR_E_INVAL : CTR_E_DEVICE);
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
