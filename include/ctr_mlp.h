/*
 * ctr_mlp.h - C ABI of the dense tower that sits between the pull and the push of the sparse
 * embedding cycle (MI355X / gfx950).
 *
 * The paper's training step is pull -> train_mini-batch -> push (Algorithm 1); the dense network
 * is a fully connected tower over the concatenated slot embeddings (Section 2.1) whose dense
 * parameters are trained with k-step Adam (Algorithm 2, Section 4; Section 5 for the setting).
 * This header covers that middle step: forward, sigmoid cross-entropy loss, backward down to the
 * gradient of the pooled embeddings (the input of ctr_push_adam), and the dense optimizer.
 *
 * Arithmetic: matrix products take bf16 operands with fp32 accumulation on the matrix cores, in
 * the library's own kernel (fixed summation order; bias + ReLU + rounding, and the ReLU gate of a
 * back-propagated gradient + rounding, are applied as the products are stored); no vendor GEMM
 * library is involved.  Master parameters, moments and the
 * optimizer are fp32/fp64 exactly as in the sparse path: m0 = 0, v0 = eps, no bias correction,
 * x -= lr m / sqrt(den) with den = own v (one replica) or the shared v frozen at the last merge.
 * Rounding to bf16 (nearest-even) happens at: the input, the weight copies used by the products,
 * every hidden activation, and every back-propagated hidden gradient.
 *
 * Conventions are those of ctr_sparse.h: d_* device pointers owned by the caller, `hip_stream`
 * a hipStream_t, calls enqueue only, status codes of ctr_status.  The tower allocates no device
 * memory of its own.
 */
#ifndef CTR_MLP_H
#define CTR_MLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ctr_mlp ctr_mlp; /* opaque host-side handle */

#define CTR_MLP_MAX_HIDDEN 6
#define CTR_MLP_MAX_BATCH (1u << 20) /* samples per call */

typedef struct {
  uint32_t in_dim;                     /* width of the input (slots x embedding dim), multiple of 8 */
  uint32_t n_hidden;                   /* 1..CTR_MLP_MAX_HIDDEN hidden ReLU layers */
  uint32_t hidden[CTR_MLP_MAX_HIDDEN]; /* their widths, multiples of 8; the output layer has width 1 */
  uint32_t n_replicas;                 /* W >= 1 model replicas (W > 1 needs kstep) */
  uint32_t kstep;                      /* 1: Algorithm 2 with a shared denominator and ctr_mlp_kstep_merge */
  float lr, beta1, beta2, eps;         /* alpha, beta_1, beta_2, epsilon of Algorithm 2 */
  uint64_t init_seed;                  /* weights: deterministic stand-in for N(0, 2 / fan_in); biases 0 */
} ctr_mlp_config;

/* Bytes of device memory for the parameters, moments and bf16 copies of all replicas (0 if the
 * configuration is invalid), and of per-step workspace for a batch of `batch` samples. */
size_t ctr_mlp_bytes(const ctr_mlp_config* cfg);
size_t ctr_mlp_workspace_bytes(const ctr_mlp_config* cfg, uint32_t batch);

/* Creates the tower in caller-provided device memory (256-byte aligned, >= ctr_mlp_bytes) and
 * enqueues the initialisation of every replica (all replicas start equal: Algorithm 2's x_0).
 * Errors: CTR_E_INVAL, CTR_E_NOMEM, CTR_E_DEVICE. */
int ctr_mlp_create(const ctr_mlp_config* cfg, void* d_mem, size_t bytes, void* hip_stream, ctr_mlp** out);
int ctr_mlp_destroy(ctr_mlp* m);

/* One training step of replica `replica` (Algorithm 1's train_mini-batch; Algorithm 2's m, v and
 * model lines on the dense parameters):
 *   d_pooled[batch * in_dim]       device, in: fp32 pooled embeddings (output of ctr_pull_pool)
 *   d_labels[batch]                device, in: fp32 0/1 click labels
 *   d_grad_pooled[batch * in_dim]  device, out: d(mean loss)/d(pooled), fp32 (input of ctr_push_adam)
 *   d_loss                         device, out: one float, the mean sigmoid cross-entropy
 *   d_workspace                    device, >= ctr_mlp_workspace_bytes(cfg, batch), 256-byte aligned
 *   mode                           CTR_STEP_LOCAL or CTR_STEP_MERGE_PENDING, as in ctr_push_adam
 * batch must be a multiple of 8 and at most CTR_MLP_MAX_BATCH.  Errors: CTR_E_INVAL, CTR_E_NOMEM, CTR_E_DEVICE. */
int ctr_mlp_step(ctr_mlp* m, uint32_t replica, const float* d_pooled, const float* d_labels, uint32_t batch,
                 float* d_grad_pooled, float* d_loss, void* d_workspace, size_t workspace_bytes, uint32_t mode,
                 void* hip_stream);

/* Forward only: d_logits[batch] fp32 (no parameter changes). */
int ctr_mlp_forward(ctr_mlp* m, uint32_t replica, const float* d_pooled, uint32_t batch, float* d_logits,
                    void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* The same two calls for an input that is already bfloat16 (d_pooled_bf16[batch * in_dim], the
 * output of ctr_pull_pool_bf16; read in place, must stay unchanged until the step's work has
 * run).  The results equal those of the fp32 calls on an input that rounds to these bf16 values. */
int ctr_mlp_step_bf16(ctr_mlp* m, uint32_t replica, const uint16_t* d_pooled_bf16, const float* d_labels,
                      uint32_t batch, float* d_grad_pooled, float* d_loss, void* d_workspace,
                      size_t workspace_bytes, uint32_t mode, void* hip_stream);
int ctr_mlp_forward_bf16(ctr_mlp* m, uint32_t replica, const uint16_t* d_pooled_bf16, uint32_t batch,
                         float* d_logits, void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ctr_mlp_step_bf16 with the gradient of the pooled embeddings written as bfloat16 too
 * (d_grad_pooled_bf16[batch * in_dim], the input of ctr_push_adam_bf16): the first layer's
 * input-gradient product rounds its fp32 sums to bf16 (nearest-even) on the way out, one more
 * rounding point beside those listed above.  Everything else is as in ctr_mlp_step_bf16. */
int ctr_mlp_step_bf16_grad_bf16(ctr_mlp* m, uint32_t replica, const uint16_t* d_pooled_bf16, const float* d_labels,
                                uint32_t batch, uint16_t* d_grad_pooled_bf16, float* d_loss, void* d_workspace,
                                size_t workspace_bytes, uint32_t mode, void* hip_stream);

/* The tower's matrix product on its own, for tests and measurements (Algorithm 1's train_mini-batch is
 * made of three of these per layer): C[m x n] (fp32, row-major, rows ldc floats apart) = A[m x k] B[k x n]
 * with bf16 operands and fp32 accumulation on the matrix cores, by the library's own kernel.
 *   a_k_contiguous != 0: A is stored as m rows of k values (rows lda apart); else as k rows of m values
 *   b_k_contiguous != 0: B is stored as n rows of k values (rows ldb apart); else as k rows of n values
 *   d_scratch: device fp32 scratch for contractions split over several workgroups (may be NULL: no
 *              split), scratch_bytes its size; the summation order is fixed either way
 * All of m, n, k, lda, ldb, ldc are multiples of 8, every pointer is 16-byte aligned, each operand holds
 * less than 4 GiB.  Enqueues only.  Errors: CTR_E_INVAL, CTR_E_DEVICE. */
int ctr_mlp_gemm(int a_k_contiguous, int b_k_contiguous, const uint16_t* d_a, uint32_t lda, const uint16_t* d_b,
                 uint32_t ldb, uint32_t m, uint32_t n, uint32_t k, float* d_c, uint32_t ldc, void* d_scratch,
                 size_t scratch_bytes, void* hip_stream);

/* Algorithm 2's global-averaging branch over all dense parameters of the W replicas:
 * shared v = mean_j v_j; x_i = mean_j (x_j - [merge step pending in j] lr m_j / sqrt(shared v)). */
int ctr_mlp_kstep_merge(ctr_mlp* m, void* hip_stream);

/* Number of parameters of one replica (weights and biases of all layers, in layer order:
 * W_1[in x h_1] row-major, b_1[h_1], W_2, b_2, ..., w_out[h_last x 1], b_out[1]). */
size_t ctr_mlp_n_params(const ctr_mlp_config* cfg);

/* Debug: copies the flat parameter vector, first and second moments of a replica and the shared
 * denominator (kstep only) to HOST arrays of ctr_mlp_n_params floats (any may be NULL);
 * synchronises the stream. */
int ctr_mlp_export(ctr_mlp* m, uint32_t replica, float* h_params, float* h_m, float* h_v, float* h_vhat,
                   void* hip_stream);

/* The inverse of ctr_mlp_export (restoring a checkpoint): copies HOST arrays of ctr_mlp_n_params
 * floats into a replica's parameters, first and second moments and into the shared denominator
 * (any may be NULL: left as it is), refreshes the bf16 copy of the parameters, and sets whether
 * the replica's last step was a merge step that the next ctr_mlp_kstep_merge still has to apply
 * (pending: 0 or 1).  Synchronises the stream.  Errors: CTR_E_INVAL, CTR_E_DEVICE. */
int ctr_mlp_import(ctr_mlp* m, uint32_t replica, const float* h_params, const float* h_m, const float* h_v,
                   const float* h_vhat, uint32_t pending, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CTR_MLP_H */
