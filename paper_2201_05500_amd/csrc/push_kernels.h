// Gradient segment-reduce by row fused with the sparse Adam update, and the k-step merge.
//
// Paper: Algorithm 1's push step (one update per referenced parameter per
// mini-batch) and Algorithm 2: the m, v and model lines, the local branch with
// the shared denominator frozen since the last merge, and the global-averaging
// branch.
//
// Input is the occurrence list sorted by row id: sr[i] = row, ss[i] = segment.
// The list is cut into spans of SPAN occurrences; a group of LPR lanes (each
// lane owns 4 columns) walks one span, summing grad[ss[i], :] in binary64.  A
// row that lies wholly inside a span is updated on the spot.  A row that
// crosses a span boundary leaves binary64 partial sums (the span where it
// starts writes a "tail", every later span it reaches writes a "head"); a
// second launch adds them up in a fixed order and updates the row.  Work per
// group is bounded by SPAN whatever the popularity of a key, and the summation
// order is fixed, so results do not depend on scheduling.
#pragma once
#include "common.h"

namespace ctr {

constexpr u32 SPAN = 128;
constexpr u32 SF_HEAD = 1u, SF_TAIL = 2u;

struct AdamParams {
  double b1, omb1, b2, omb2;  // beta and (1 - beta) promoted from binary32
  float lr;
  u32 mode;      // 0: den = own v   1: den = shared denominator   2: moments only (merge pending)
  u32 kstep;     // maintain the per-row state word
  u32 pend_bit;  // (1 << replica) when mode == 2, else 0
};

// One Adam step on 4 columns of one row.  m and v are formed in binary64 from
// the stored binary32 values and rounded once; the model step is binary32 with
// correctly rounded sqrt and divide.
__device__ __forceinline__ void adam_row4(float* __restrict__ row_base, const float* __restrict__ vhat_row,
                                          u32 D, u32 c, d4 g, const AdamParams& P) {
  float* px = row_base + 4 * c;
  f4 x = ldg4(px), m = ldg4(px + D), v = ldg4(px + 2 * D);
  m.x = (float)(P.b1 * (double)m.x + P.omb1 * g.x);
  m.y = (float)(P.b1 * (double)m.y + P.omb1 * g.y);
  m.z = (float)(P.b1 * (double)m.z + P.omb1 * g.z);
  m.w = (float)(P.b1 * (double)m.w + P.omb1 * g.w);
  v.x = (float)(P.b2 * (double)v.x + P.omb2 * (g.x * g.x));
  v.y = (float)(P.b2 * (double)v.y + P.omb2 * (g.y * g.y));
  v.z = (float)(P.b2 * (double)v.z + P.omb2 * (g.z * g.z));
  v.w = (float)(P.b2 * (double)v.w + P.omb2 * (g.w * g.w));
  stg4(px + D, m);
  stg4(px + 2 * D, v);
  if (P.mode != 2u) {
    f4 den = v;
    if (P.mode == 1u) den = ldg4(vhat_row + 4 * c);
    x.x = x.x - P.lr * (m.x / sqrtf(den.x));
    x.y = x.y - P.lr * (m.y / sqrtf(den.y));
    x.z = x.z - P.lr * (m.z / sqrtf(den.z));
    x.w = x.w - P.lr * (m.w / sqrtf(den.w));
    stg4(px, x);
  }
}

__device__ __forceinline__ void finish_row(u32 row, d4 g, u32 c, bool col_ok, float* __restrict__ values,
                                           const float* __restrict__ vhat, u32* __restrict__ row_state, u32 D,
                                           const AdamParams& P) {
  if (col_ok) adam_row4(values + (u64)row * 3 * D, vhat ? vhat + (u64)row * D : nullptr, D, c, g, P);
  if (P.kstep && c == 0) atomicOr(&row_state[row], RS_TOUCHED | P.pend_bit);
}

template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_push_span(const DevHeader* hdr, const u32* __restrict__ sr, const u32* __restrict__ ss, u32 n,
            const float* __restrict__ grad, float* __restrict__ values, const float* __restrict__ vhat,
            u32* __restrict__ row_state, u32 D, AdamParams P, double* __restrict__ head_part,
            double* __restrict__ tail_part, u32* __restrict__ span_flags, u32* __restrict__ span_rows) {
  if (hdr->status) return;
  const u32 s = (blockIdx.x * BLOCK + threadIdx.x) / LPR;
  const u32 c = threadIdx.x % LPR;
  const u32 b = s * SPAN;
  if (b >= n) return;
  const u32 e = min(b + SPAN, n);
  const bool col_ok = c * 4 < D;

  u32 cur = sr[b];
  bool open_left = (b > 0) && (sr[b - 1] == cur);
  u32 flags = 0, finished = 0;
  d4 acc = {0.0, 0.0, 0.0, 0.0};

  for (u32 i0 = b; i0 < e; i0 += 4) {
    u32 r[4], g[4];
    f4 gv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = i0 + i < e;
      r[i] = ok ? sr[i0 + i] : cur;
      g[i] = ok ? ss[i0 + i] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      gv[i].x = gv[i].y = gv[i].z = gv[i].w = 0.0f;
      if (i0 + i < e && col_ok) gv[i] = ldg4(grad + (u64)g[i] * D + 4 * c);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i0 + i < e) {
        if (r[i] != cur) {  // the row `cur` ends here
          if (open_left) {
            if (col_ok) {
              double* hp = head_part + ((u64)s * D + 4 * c);
              hp[0] = acc.x; hp[1] = acc.y; hp[2] = acc.z; hp[3] = acc.w;
            }
            flags |= SF_HEAD;
            open_left = false;
          } else {
            finish_row(cur, acc, c, col_ok, values, vhat, row_state, D, P);
            ++finished;
          }
          cur = r[i];
          acc.x = acc.y = acc.z = acc.w = 0.0;
        }
        acc.x += (double)gv[i].x;
        acc.y += (double)gv[i].y;
        acc.z += (double)gv[i].z;
        acc.w += (double)gv[i].w;
      }
    }
  }

  const bool open_right = (e < n) && (sr[e] == cur);
  if (open_left) {  // the whole span belongs to a row that began earlier
    if (col_ok) {
      double* hp = head_part + ((u64)s * D + 4 * c);
      hp[0] = acc.x; hp[1] = acc.y; hp[2] = acc.z; hp[3] = acc.w;
    }
    flags |= SF_HEAD;
  } else if (open_right) {  // the row began in this span and goes on
    if (col_ok) {
      double* tp = tail_part + ((u64)s * D + 4 * c);
      tp[0] = acc.x; tp[1] = acc.y; tp[2] = acc.z; tp[3] = acc.w;
    }
    flags |= SF_TAIL;
  } else {
    finish_row(cur, acc, c, col_ok, values, vhat, row_state, D, P);
    ++finished;
  }
  if (c == 0) {
    span_flags[s] = flags;
    span_rows[s] = finished + ((flags & SF_TAIL) ? 1u : 0u);  // rows that START in this span
  }
}

// One wave per span that holds a tail: adds the tail and the heads of the
// following spans that continue the same row (its groups take the spans in
// turn, then combine), and updates the row.
template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_push_fixup(const DevHeader* hdr, const u32* __restrict__ sr, u32 n, u32 n_spans, float* __restrict__ values,
             const float* __restrict__ vhat, u32* __restrict__ row_state, u32 D, AdamParams P,
             const double* __restrict__ head_part, const double* __restrict__ tail_part,
             const u32* __restrict__ span_flags) {
  if (hdr->status) return;
  constexpr int GPW = WAVE / LPR;
  const u32 s = (blockIdx.x * BLOCK + threadIdx.x) / WAVE;  // wave-uniform
  if (s >= n_spans) return;
  if (!(span_flags[s] & SF_TAIL)) return;
  const int lane = lane_id();
  const u32 c = lane % LPR;
  const u32 grp = lane / LPR;
  const bool col_ok = c * 4 < D;
  const u32 row = sr[min((s + 1) * SPAN, n) - 1];

  d4 acc = {0.0, 0.0, 0.0, 0.0};
  if (grp == 0 && col_ok) {
    const double* tp = tail_part + ((u64)s * D + 4 * c);
    acc.x = tp[0]; acc.y = tp[1]; acc.z = tp[2]; acc.w = tp[3];
  }
  for (u32 t = s + 1 + grp; t < n_spans; t += GPW) {
    if (sr[t * SPAN] != row) break;
    if (col_ok) {
      const double* hp = head_part + ((u64)t * D + 4 * c);
      acc.x += hp[0]; acc.y += hp[1]; acc.z += hp[2]; acc.w += hp[3];
    }
  }
#pragma unroll
  for (int off = LPR; off < WAVE; off <<= 1) {
    acc.x += __shfl_xor(acc.x, off, WAVE);
    acc.y += __shfl_xor(acc.y, off, WAVE);
    acc.z += __shfl_xor(acc.z, off, WAVE);
    acc.w += __shfl_xor(acc.w, off, WAVE);
  }
  if (grp == 0) finish_row(row, acc, c, col_ok, values, vhat, row_state, D, P);
}

// Sum of the per-span counts of rows that start in the span = distinct keys of the batch.
// The counter is zeroed by the pull (k_scan_tiles).
__global__ void k_count_unique(DevHeader* hdr, const u32* __restrict__ span_rows, u32 n_spans) {
  if (hdr->status) return;
  __shared__ u32 lds[4];
  u32 s = 0;
  for (u32 i = blockIdx.x * BLOCK + threadIdx.x; i < n_spans; i += gridDim.x * BLOCK) s += span_rows[i];
  u32 total;
  block_exclusive_scan(s, lds, total);
  if (threadIdx.x == 0 && total) atomicAdd(&hdr->n_unique, total);
}

// k-step merge.  One group of LPR lanes per row in use; rows nobody touched
// since the last merge are skipped.  vhat = mean_j v_j; every replica's x becomes
// mean_j (x_j - [pending_j] lr m_j / sqrt(vhat)); sums in binary64, rounded once.
template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_merge(const DevHeader* hdr, float* __restrict__ values, u64 replica_stride, u32 W, float* __restrict__ vhat,
        u32* __restrict__ row_state, u32 D, float lr) {
  if (hdr->status) return;
  const u32 n_rows = hdr->n_rows;
  const u32 c = threadIdx.x % LPR;
  const u32 groups = gridDim.x * (BLOCK / LPR);
  const bool col_ok = c * 4 < D;
  for (u32 row = (blockIdx.x * BLOCK + threadIdx.x) / LPR; row < n_rows; row += groups) {
    const u32 st = row_state[row];
    if (!(st & RS_TOUCHED)) continue;
    if (col_ok) {
      float* base = values + (u64)row * 3 * D + 4 * c;
      d4 vs = {0.0, 0.0, 0.0, 0.0};
      for (u32 j = 0; j < W; ++j) {
        const f4 v = ldg4(base + j * replica_stride + 2 * D);
        vs.x += (double)v.x; vs.y += (double)v.y; vs.z += (double)v.z; vs.w += (double)v.w;
      }
      const double w = (double)W;
      f4 vh;
      vh.x = (float)(vs.x / w); vh.y = (float)(vs.y / w); vh.z = (float)(vs.z / w); vh.w = (float)(vs.w / w);
      stg4(vhat + (u64)row * D + 4 * c, vh);
      f4 den;
      den.x = sqrtf(vh.x); den.y = sqrtf(vh.y); den.z = sqrtf(vh.z); den.w = sqrtf(vh.w);
      d4 xs = {0.0, 0.0, 0.0, 0.0};
      for (u32 j = 0; j < W; ++j) {
        const f4 x = ldg4(base + j * replica_stride);
        d4 y = {(double)x.x, (double)x.y, (double)x.z, (double)x.w};
        if (st & (1u << j)) {
          const f4 m = ldg4(base + j * replica_stride + D);
          y.x -= (double)(lr * (m.x / den.x));
          y.y -= (double)(lr * (m.y / den.y));
          y.z -= (double)(lr * (m.z / den.z));
          y.w -= (double)(lr * (m.w / den.w));
        }
        xs.x += y.x; xs.y += y.y; xs.z += y.z; xs.w += y.w;
      }
      f4 xb;
      xb.x = (float)(xs.x / w); xb.y = (float)(xs.y / w); xb.z = (float)(xs.z / w); xb.w = (float)(xs.w / w);
      for (u32 j = 0; j < W; ++j) stg4(base + j * replica_stride, xb);
    }
    if (c == 0) row_state[row] = 0;
  }
}

}  // namespace ctr
