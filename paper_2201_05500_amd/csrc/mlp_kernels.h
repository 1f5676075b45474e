// Element-wise and reduction kernels of the dense tower (the matrix products, with bias + ReLU and the
// ReLU gate of back-propagated gradients fused into their epilogues, are in gemm_kernels.h).
//
// Paper: the train_mini-batch step of Algorithm 1 on the network of Section 2.1, and Algorithm 2
// (k-step Adam) on the dense parameters.  bf16 rounding is nearest-even, done here by hand so that
// it is the same rule everywhere: (u + 0x7FFF + ((u >> 16) & 1)) >> 16 on the fp32 bit pattern.
#pragma once
#include "common.h"

namespace ctr {

struct MlpLayout {
  u32 n_layers;        // hidden layers + the output layer
  u32 in[8], out[8];   // widths per layer
  u64 w_off[8];        // offset of W_l in the flat parameter vector (b_l follows W_l)
  u64 n_params;
};

// fp32 -> bf16, 4 values per thread (n multiple of 4).
__global__ void k_cast_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, u64 n) {
  const u64 i = ((u64)blockIdx.x * BLOCK + threadIdx.x) * 4;
  if (i >= n) return;
  const f4 v = ldg4(src + i);
  ushort4 o;
  o.x = to_bf16(v.x); o.y = to_bf16(v.y); o.z = to_bf16(v.z); o.w = to_bf16(v.w);
  *reinterpret_cast<ushort4*>(dst + i) = o;
}

// Output layer (width 1): logit[b] = a[b, :] . w + bias.  One wave per sample, fixed summation order.
__global__ void k_out_forward(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w, const float* __restrict__ bias,
                              u32 rows, u32 H, float* __restrict__ logits) {
  const u32 r = (blockIdx.x * BLOCK + threadIdx.x) / WAVE;
  if (r >= rows) return;
  const int lane = lane_id();
  float s = 0.0f;
  for (u32 j = lane; j < H; j += WAVE) s += from_bf16(a[(u64)r * H + j]) * from_bf16(w[j]);
#pragma unroll
  for (int off = WAVE / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, WAVE);
  if (lane == 0) logits[r] = s + bias[0];
}

// Sigmoid cross-entropy with logits, evaluated in binary64 per sample:
// lterm[b] = max(z, 0) - z y + log1p(exp(-|z|)) and dlogit[b] = (sigmoid(z) - y) / rows.
__global__ void k_bce(const float* __restrict__ logits, const float* __restrict__ labels, u32 rows,
                      float* __restrict__ dlogit, double* __restrict__ lterm) {
  const u32 r = blockIdx.x * BLOCK + threadIdx.x;
  if (r >= rows) return;
  const double z = (double)logits[r], y = (double)labels[r];
  lterm[r] = fmax(z, 0.0) - z * y + log1p(exp(-fabs(z)));
  dlogit[r] = (float)((1.0 / (1.0 + exp(-z)) - y) / (double)rows);
}

// Mean of the per-sample loss terms, summed by ONE block in a fixed order.
__global__ void k_loss_mean(const double* __restrict__ lterm, u32 rows, float* __restrict__ loss) {
  __shared__ double part[BLOCK];
  double s = 0.0;
  for (u32 r = threadIdx.x; r < rows; r += BLOCK) s += lterm[r];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = BLOCK / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(part[0] / (double)rows);
}

// Back through the output layer and the last ReLU: dz[b, j] = bf16(dlogit[b] * w[j] * [a[b, j] > 0]).
__global__ void k_out_backward_dz(const bf16_t* __restrict__ a, const float* __restrict__ dlogit,
                                  const bf16_t* __restrict__ w, u32 H, u64 n, bf16_t* __restrict__ dz) {
  const u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  if (i >= n) return;
  const u32 j = (u32)(i % H);
  const float av = from_bf16(a[i]);
  dz[i] = to_bf16(av > 0.0f ? dlogit[i / H] * from_bf16(w[j]) : 0.0f);
}

// Column sums over the batch in a fixed order: out[j] = sum_b x[b, j] * (wgt ? wgt[b] : 1).
// Stage 1: block (column tile of 32, row slice) - its 8 row groups each sum the slice's rows
// congruent to them, the 8 partial sums are added in order -> partial[slice][column].
// Stage 2: the slices are added in order.  Used for bias gradients and the output layer's weights.
constexpr u32 COLSUM_SLICES = 64;

__global__ void k_colsum_partial(const bf16_t* __restrict__ x, const float* __restrict__ wgt, u32 rows, u32 H,
                                 float* __restrict__ partial) {
  __shared__ float part[8][32];
  const u32 col = blockIdx.x * 32 + (threadIdx.x & 31);
  const u32 rg = threadIdx.x >> 5;
  const u32 per = (rows + COLSUM_SLICES - 1) / COLSUM_SLICES;
  const u32 r0 = blockIdx.y * per, r1 = min(r0 + per, rows);
  float s = 0.0f;
  if (col < H)
    for (u32 r = r0 + rg; r < r1; r += 8) s += from_bf16(x[(u64)r * H + col]) * (wgt ? wgt[r] : 1.0f);
  part[rg][threadIdx.x & 31] = s;
  __syncthreads();
  if (rg == 0 && col < H) {
    float t = part[0][threadIdx.x];
#pragma unroll
    for (int g = 1; g < 8; ++g) t += part[g][threadIdx.x];
    partial[(u64)blockIdx.y * H + col] = t;
  }
}

__global__ void k_colsum_final(const float* __restrict__ partial, u32 H, float* __restrict__ out) {
  const u32 col = blockIdx.x * BLOCK + threadIdx.x;
  if (col >= H) return;
  float t = 0.0f;
  for (u32 sl = 0; sl < COLSUM_SLICES; ++sl) t += partial[(u64)sl * H + col];
  out[col] = t;
}

// Sum of a vector (the output bias gradient = sum of dlogit), one block, fixed order.
__global__ void k_sum_f32(const float* __restrict__ x, u32 n, float* __restrict__ out) {
  __shared__ float part[BLOCK];
  float s = 0.0f;
  for (u32 i = threadIdx.x; i < n; i += BLOCK) s += x[i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = BLOCK / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = part[0];
}

// Initial parameters of every replica: weights from the integer recipe of the row initialiser with
// key = layer << 48 | index, scaled to a standard deviation of sqrt(2 / fan_in); biases 0; m = 0;
// v = shared v = eps (Algorithm 2, "Initialize"); bf16 copies of the parameters.
__global__ void k_mlp_init(MlpLayout L, u64 seed_mul, float eps, u32 W, u64 stride, float* __restrict__ params,
                           float* __restrict__ m, float* __restrict__ v, float* __restrict__ vhat,
                           bf16_t* __restrict__ pb) {
  const u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  if (i >= L.n_params) return;
  float val = 0.0f;
  for (u32 l = 0; l < L.n_layers; ++l) {
    const u64 nw = (u64)L.in[l] * L.out[l];
    if (i >= L.w_off[l] && i < L.w_off[l] + nw) {
      const float scale = (float)(sqrt(2.0 / (double)L.in[l]) / 37837.2);
      val = init_value(seed_mul, ((u64)l << 48) | (i - L.w_off[l]), 0, scale);
    }
  }
  for (u32 j = 0; j < W; ++j) {
    params[j * stride + i] = val;
    m[j * stride + i] = 0.0f;
    v[j * stride + i] = eps;
    pb[j * stride + i] = to_bf16(val);
  }
  if (vhat) vhat[i] = eps;
}

// bf16 copy of a flat fp32 vector (any length).
__global__ void k_refresh_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, u64 n) {
  const u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  if (i < n) dst[i] = to_bf16(src[i]);
}

// Dense Adam step (Algorithm 2's m, v and model lines) on one replica's flat parameter vector;
// every assignment in binary64 from the stored fp32 values, rounded once; refreshes the bf16 copy.
//   mode 0: x -= lr m / sqrt(own v)   1: x -= lr m / sqrt(shared v)   2: moments only (merge pending)
__global__ void k_dense_adam(float* __restrict__ params, float* __restrict__ m, float* __restrict__ v,
                             const float* __restrict__ vhat, const float* __restrict__ grad,
                             bf16_t* __restrict__ pb, u64 n, double b1, double b2, double lr, u32 mode) {
  const u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  if (i >= n) return;
  const double g = (double)grad[i];
  const float mn = (float)(b1 * (double)m[i] + (1.0 - b1) * g);
  const float vn = (float)(b2 * (double)v[i] + (1.0 - b2) * (g * g));
  m[i] = mn;
  v[i] = vn;
  if (mode != 2u) {
    const double den = (double)(mode == 1u ? vhat[i] : vn);
    const float xn = (float)((double)params[i] - lr * (double)mn / sqrt(den));
    params[i] = xn;
    pb[i] = to_bf16(xn);
  }
}

// Algorithm 2's global-averaging branch on the dense parameters of W replicas.
__global__ void k_dense_merge(float* __restrict__ params, const float* __restrict__ m, const float* __restrict__ v,
                              float* __restrict__ vhat, bf16_t* __restrict__ pb, u64 n, u64 stride, u32 W,
                              u32 pend_mask, double lr) {
  const u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  if (i >= n) return;
  double vs = 0.0;
  for (u32 j = 0; j < W; ++j) vs += (double)v[j * stride + i];
  const float vh = (float)(vs / (double)W);
  vhat[i] = vh;
  const double den = sqrt((double)vh);
  double xs = 0.0;
  for (u32 j = 0; j < W; ++j) {
    double y = (double)params[j * stride + i];
    if (pend_mask & (1u << j)) y -= lr * (double)m[j * stride + i] / den;
    xs += y;
  }
  const float xb = (float)(xs / (double)W);
  const bf16_t hb = to_bf16(xb);
  for (u32 j = 0; j < W; ++j) {
    params[j * stride + i] = xb;
    pb[j * stride + i] = hb;
  }
}

}  // namespace ctr
