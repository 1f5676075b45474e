// Gradient segment-reduce by row fused with the sparse Adam update, and the k-step merge.
//
// Paper: Algorithm 1's push step (one update per referenced parameter per
// mini-batch) and Algorithm 2: the m, v and model lines, the local branch with
// the shared denominator frozen since the last merge, and the global-averaging
// branch.
//
// Input is the occurrence list sorted by row id: sr[i] = row, ss[i] = segment.
// The list is cut into spans of `span` occurrences (chosen by the host from the batch size); a group of LPR lanes (each
// lane owns 4 columns) walks one span, summing grad[ss[i], :] in binary64.  A
// row that lies wholly inside a span is updated on the spot.  A row that
// crosses a span boundary leaves binary64 partial sums (the span where it
// starts writes a "tail", every later span it reaches writes a "head").  Heads
// of runs of spans that continue one row are pre-summed per block of
// SPANS_PER_BLOCK spans, and a last launch adds tail + heads + block sums in a
// fixed order and updates the row.  Work per group is bounded by the span whatever
// the popularity of a key, and the summation order is fixed, so results do not
// depend on scheduling.
#pragma once
#include "common.h"

namespace ctr {

constexpr u32 MAX_SPAN = 128;  // spans are 16..128 occurrences: shorter for small batches, to keep the chip busy
constexpr u32 SPANS_PER_BLOCK = 64;  // one wave lane per span when scanning a block
constexpr u32 SF_HEAD = 1u, SF_TAIL = 2u;
constexpr u32 NO_ROW = 0xFFFFFFFFu;
#ifndef CTR_PUSH_PB
#define CTR_PUSH_PB 2  // occurrences per batch of the span walk (2: 71 VGPRs, 7 waves/SIMD; measured best)
#endif
// cache hints of the span walk's three traffic classes (0 = plain access, 1 = non-temporal)
#ifndef CTR_PUSH_NT_GRAD
#define CTR_PUSH_NT_GRAD 0
#endif
#ifndef CTR_PUSH_NT_ROW_LD
#define CTR_PUSH_NT_ROW_LD 1
#endif
#ifndef CTR_PUSH_NT_ROW_ST
#define CTR_PUSH_NT_ROW_ST 1
#endif
#ifndef CTR_MERGE_MB
#define CTR_MERGE_MB 8  // replicas whose loads the merge issues together
#endif
#ifndef CTR_PUSH_MIN_WAVES
#define CTR_PUSH_MIN_WAVES 1  // waves per SIMD the span kernel is compiled for
#endif
// Execution order of the spans (initial values; ctr_debug_set_push_order changes them per table).
// CTR_PUSH_WINDOWS > 0 (a power of two up to 128): the spans that lie inside one row - pure gradient gathers,
// in ascending segment order - are run first, grouped by which of that many windows of the gradient array
// they begin in, so that the spans in flight at one time gather from one window and the second use of a
// gradient row finds it in the last-level cache; the other spans follow in list order.  Only the order of
// execution changes: every span still writes its own partial sums.  0: list order.
#ifndef CTR_PUSH_WINDOWS
#define CTR_PUSH_WINDOWS 32
#endif
// 0: one launch, those spans first.  1: they get a launch of their own (k_push_hot: nothing but gathers and
// one partial sum per span, CTR_PUSH_HOT_PB gradient rows in flight per lane group), the rest a second one.
// 2: one launch, the other spans dealt evenly between the windows.  (Measured: 0 and 2 equal, 1 slower.)
#ifndef CTR_PUSH_SPLIT
#define CTR_PUSH_SPLIT 0
#endif
#ifndef CTR_PUSH_HOT_PB
#define CTR_PUSH_HOT_PB 8
#endif
// a gradient array smaller than this many bytes stays in the last-level cache whatever the order: its
// pushes keep the list order (and save the four short launches that compute the other one)
#ifndef CTR_PUSH_ORDER_MIN_GRAD_BYTES
#define CTR_PUSH_ORDER_MIN_GRAD_BYTES (256ull << 20)
#endif

// Which row update a launch performs (compile-time, so that each variant carries only its own
// registers and loads).
enum StepKind : int {
  STEP_ADAM_OWN = 0,     // Algorithm 2's m/v lines, step divided by the row's own v (single table, or the
                         // "standard Adam locally" reading of Section 4); also the moments-only merge step
  STEP_ADAM_SHARED = 1,  // Algorithm 2 local branch: step divided by the shared v frozen at the last merge
  STEP_ADAGRAD = 2,      // the paper's production optimizer for sparse parameters (Section 5): rows [x | G]
  STEP_ADAM_KINGMA = 3   // the cited Adam of Kingma & Ba: bias-corrected moments, eps added to the root
};

struct AdamParams {
  double b1, omb1, b2, omb2;  // beta and (1 - beta) promoted from binary32
  double bc1, bc2, eps;       // STEP_ADAM_KINGMA: 1/(1 - beta1^t), 1/(1 - beta2^t) (filled in on the device from
                              // the header), epsilon
  float lr;
  u32 mode;      // 0: moments and model   2: moments only (merge pending)
  u32 kstep;     // maintain the per-row state word
  u32 pend_bit;  // (1 << replica) when mode == 2, else 0
};

struct RowState4 {
  f4 x, m, v, den;  // v doubles as AdaGrad's accumulator; den: shared denominator (STEP_ADAM_SHARED only)
};

__device__ __forceinline__ f4 row_ld4(const float* p) {
#if CTR_PUSH_NT_ROW_LD
  return ldg4_stream(p);
#else
  return ldg4(p);
#endif
}
__device__ __forceinline__ void row_st4(float* p, f4 v) {
#if CTR_PUSH_NT_ROW_ST
  stg4_stream(p, v);
#else
  stg4(p, v);
#endif
}

// rf = floats per row: 3*D for [x | m | v], 2*D for AdaGrad's [x | G].
template <int KIND>
__device__ __forceinline__ RowState4 load_row4(const float* __restrict__ values, const float* __restrict__ vhat,
                                               u32 row, u32 D, u32 rf, u32 c) {
  RowState4 s;
  const float* px = values + (u64)row * rf + 4 * c;
  s.x = row_ld4(px);
  if constexpr (KIND == STEP_ADAGRAD) {
    s.v = row_ld4(px + D);
  } else {
    s.m = row_ld4(px + D);
    s.v = row_ld4(px + 2 * D);
  }
  if constexpr (KIND == STEP_ADAM_SHARED) s.den = ldg4(vhat + (u64)row * D + 4 * c);
  return s;
}

__device__ __forceinline__ double rsqrt_refined(float a) {
  const double y = (double)rsqrtf(a), d = (double)a;
  return y * (1.5 - 0.5 * d * y * y);
}

// One optimizer step on 4 columns of one row whose state is already in registers.  Every
// assignment is evaluated in binary64 from the stored binary32 values and rounded once.
// A binary32 quotient for the model step would leave an error proportional to the step, which
// can be orders of magnitude larger than the parameter it lands on (shared denominator still at
// eps); 1/sqrt(den) is a binary32 estimate refined by one Newton step in binary64 (relative error
// ~1e-13), cheaper than a binary64 sqrt and divide.
template <int KIND>
__device__ __forceinline__ void row_apply4(RowState4 s, float* __restrict__ row_base, u32 D, u32 c, d4 g,
                                           const AdamParams& P) {
  float* px = row_base + 4 * c;
  f4 x = s.x, m = s.m, v = s.v;
  const double lr = (double)P.lr;
  if constexpr (KIND == STEP_ADAGRAD) {
    v.x = (float)((double)v.x + g.x * g.x);
    v.y = (float)((double)v.y + g.y * g.y);
    v.z = (float)((double)v.z + g.z * g.z);
    v.w = (float)((double)v.w + g.w * g.w);
    row_st4(px + D, v);
    x.x = (float)((double)x.x - lr * g.x * rsqrt_refined(v.x));
    x.y = (float)((double)x.y - lr * g.y * rsqrt_refined(v.y));
    x.z = (float)((double)x.z - lr * g.z * rsqrt_refined(v.z));
    x.w = (float)((double)x.w - lr * g.w * rsqrt_refined(v.w));
    row_st4(px, x);
    return;
  }
  m.x = (float)(P.b1 * (double)m.x + P.omb1 * g.x);
  m.y = (float)(P.b1 * (double)m.y + P.omb1 * g.y);
  m.z = (float)(P.b1 * (double)m.z + P.omb1 * g.z);
  m.w = (float)(P.b1 * (double)m.w + P.omb1 * g.w);
  v.x = (float)(P.b2 * (double)v.x + P.omb2 * (g.x * g.x));
  v.y = (float)(P.b2 * (double)v.y + P.omb2 * (g.y * g.y));
  v.z = (float)(P.b2 * (double)v.z + P.omb2 * (g.z * g.z));
  v.w = (float)(P.b2 * (double)v.w + P.omb2 * (g.w * g.w));
  row_st4(px + D, m);
  row_st4(px + 2 * D, v);
  if constexpr (KIND == STEP_ADAM_KINGMA) {
    x.x = (float)((double)x.x - lr * ((double)m.x * P.bc1) / (sqrt((double)v.x * P.bc2) + P.eps));
    x.y = (float)((double)x.y - lr * ((double)m.y * P.bc1) / (sqrt((double)v.y * P.bc2) + P.eps));
    x.z = (float)((double)x.z - lr * ((double)m.z * P.bc1) / (sqrt((double)v.z * P.bc2) + P.eps));
    x.w = (float)((double)x.w - lr * ((double)m.w * P.bc1) / (sqrt((double)v.w * P.bc2) + P.eps));
    row_st4(px, x);
  } else if (P.mode != 2u) {
    f4 den = v;
    if constexpr (KIND == STEP_ADAM_SHARED) den = s.den;
    x.x = (float)((double)x.x - lr * (double)m.x * rsqrt_refined(den.x));
    x.y = (float)((double)x.y - lr * (double)m.y * rsqrt_refined(den.y));
    x.z = (float)((double)x.z - lr * (double)m.z * rsqrt_refined(den.z));
    x.w = (float)((double)x.w - lr * (double)m.w * rsqrt_refined(den.w));
    row_st4(px, x);
  }
}

template <int KIND>
__device__ __forceinline__ void finish_row_loaded(u32 row, RowState4 s, d4 g, u32 c, bool col_ok,
                                                  float* __restrict__ values, u32* __restrict__ row_state, u32 D,
                                                  u32 rf, const AdamParams& P) {
  if (col_ok) row_apply4<KIND>(s, values + (u64)row * rf, D, c, g, P);
  if (P.kstep && c == 0) atomicOr(&row_state[row], RS_TOUCHED | P.pend_bit);
}

__device__ __forceinline__ void store_partial(double* __restrict__ part, u32 s, u32 D, u32 c, d4 a) {
  double* p = part + ((u64)s * D + 4 * c);
  p[0] = a.x; p[1] = a.y; p[2] = a.z; p[3] = a.w;
}

__device__ __forceinline__ void add_partial(const double* __restrict__ part, u32 s, u32 D, u32 c, d4& a) {
  const double* p = part + ((u64)s * D + 4 * c);
  a.x += p[0]; a.y += p[1]; a.z += p[2]; a.w += p[3];
}

// First launch of a push under the bias-corrected update: counts the push (only if the table accepts it:
// while a deferred error is pending every push is a no-op and must not advance the step count) and
// leaves the two correction factors of step t in the header for the row-update launches that follow.
__global__ void k_push_begin(DevHeader* hdr, double b1, double b2) {
  if (threadIdx.x != 0 || blockIdx.x != 0 || hdr->status) return;
  const u32 t = ++hdr->n_push;
  hdr->bc1 = 1.0 / (1.0 - pow(b1, (double)t));
  hdr->bc2 = 1.0 / (1.0 - pow(b2, (double)t));
}

// Sort key of a span for the windowed execution order: the window of the gradient array its first
// occurrence gathers from if the whole span belongs to one row, one past the last window otherwise.
__global__ void k_span_keys(const DevHeader* hdr, const u32* __restrict__ sr, const u32* __restrict__ ss, u32 n,
                            u32 span, u32 n_spans, u32 seg_shift, u32 n_windows, u32 interleave,
                            u32* __restrict__ key, u32* __restrict__ val) {
  if (hdr->status) return;
  const u32 s = blockIdx.x * BLOCK + threadIdx.x;
  if (s >= n_spans) return;
  const u32 b = s * span, e = min(b + span, n);
  // one row only, and not the whole of it: the span leaves exactly one partial sum
  const bool hot = sr[b] == sr[e - 1] && ((b > 0 && sr[b - 1] == sr[b]) || (e < n && sr[e] == sr[b]));
  const u32 w = min(ss[b] >> seg_shift, n_windows - 1u);
  if (interleave)  // the other spans are dealt evenly, by list position, between the windows
    key[s] = hot ? 2u * w : 2u * (u32)(((u64)s * n_windows) / n_spans) + 1u;
  else
    key[s] = hot ? w : n_windows;
  val[s] = s;
}

// The spans k_span_keys gave a window (the first n_spans - cold_count[0] of `order`): sum of the span's
// gradient rows in list order, left as the head (the row began in an earlier span) or the tail partial.
template <int LPR, bool GB>
__device__ __forceinline__ void push_hot_body(const DevHeader* hdr, const u32* __restrict__ sr,
                                              const u32* __restrict__ ss, u32 n, u32 span,
                                              const void* __restrict__ grad_any, u32 D,
                                              double* __restrict__ head_part, double* __restrict__ tail_part,
                                              u32* __restrict__ span_flags, u32* __restrict__ span_rows,
                                              const u32* __restrict__ order, const u32* __restrict__ cold_count) {
  if (hdr->status) return;
  constexpr int PB = CTR_PUSH_HOT_PB < LPR ? CTR_PUSH_HOT_PB : LPR;
  const u32 n_spans = (n + span - 1) / span;
  const u32 idx = (blockIdx.x * BLOCK + threadIdx.x) / LPR;
  if (idx >= n_spans - min(cold_count[0], n_spans)) return;
  const u32 s = order[idx];
  if (s >= n_spans) return;
  const u32 c = threadIdx.x % LPR;
  const u32 b = s * span, e = min(b + span, n);
  const bool col_ok = c * 4 < D;
  d4 acc = {0.0, 0.0, 0.0, 0.0};
  for (u32 i0 = b; i0 < e; i0 += LPR) {  // lane c holds the segment of list entry i0 + c
    const u32 mine = (i0 + c < e) ? ss[i0 + c] : 0u;
    const u32 cnt = min((u32)LPR, e - i0);
#pragma unroll
    for (u32 j0 = 0; j0 < (u32)LPR; j0 += PB) {
      f4 gv[PB];
#pragma unroll
      for (int j = 0; j < PB; ++j) {
        const u32 g = __shfl(mine, (int)(j0 + j), LPR);
        gv[j].x = gv[j].y = gv[j].z = gv[j].w = 0.0f;
        if (j0 + j < cnt && col_ok) {
          if constexpr (GB) {
            const uint2 raw = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(grad_any) + (u64)g * D + 4 * c);
            gv[j].x = __uint_as_float(raw.x << 16);
            gv[j].y = __uint_as_float(raw.x & 0xFFFF0000u);
            gv[j].z = __uint_as_float(raw.y << 16);
            gv[j].w = __uint_as_float(raw.y & 0xFFFF0000u);
          } else {
            gv[j] = ldg4(static_cast<const float*>(grad_any) + (u64)g * D + 4 * c);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < PB; ++j) {
        acc.x += (double)gv[j].x;
        acc.y += (double)gv[j].y;
        acc.z += (double)gv[j].z;
        acc.w += (double)gv[j].w;
      }
    }
  }
  const bool open = b > 0 && sr[b - 1] == sr[b];
  if (col_ok) store_partial(open ? head_part : tail_part, s, D, c, acc);
  if (c == 0) {
    span_flags[s] = (sr[b] << 2) | (open ? SF_HEAD : SF_TAIL);
    span_rows[s] = open ? 0u : 1u;
  }
}

// Span walk.  Each batch of PB occurrences issues, before anything is consumed,
// the PB gradient-row loads and the x/m/v loads of every row that ends inside
// the batch, so that a group keeps several KB in flight instead of one
// dependent row at a time.
// GB: the gradient rows are bf16 (two bytes per component, widened exactly) instead of fp32.
template <int LPR, int KIND, bool GB>
__device__ __forceinline__ void push_span_body(const DevHeader* hdr, const u32* __restrict__ sr,
                                               const u32* __restrict__ ss, u32 n, u32 span,
                                               const void* __restrict__ grad_any, float* __restrict__ values,
                                               const float* __restrict__ vhat, u32* __restrict__ row_state, u32 D,
                                               u32 rf, const AdamParams& P_in, double* __restrict__ head_part,
                                               double* __restrict__ tail_part, u32* __restrict__ span_flags,
                                               u32* __restrict__ span_rows, const u32* __restrict__ order,
                                               const u32* __restrict__ cold_count) {
  if (hdr->status) return;
  AdamParams P = P_in;
  if constexpr (KIND == STEP_ADAM_KINGMA) {
    P.bc1 = hdr->bc1;
    P.bc2 = hdr->bc2;
  }
  constexpr int PB = CTR_PUSH_PB;
  u32 s = (blockIdx.x * BLOCK + threadIdx.x) / LPR;
  if (order) {  // the spans are run in the order of this permutation of their indices ...
    const u32 n_spans = (n + span - 1) / span;
    u32 skip = 0;
    if (cold_count) {  // ... of which only the last cold_count[0] are this launch's
      const u32 n_cold = min(cold_count[0], n_spans);
      if (s >= n_cold) return;
      skip = n_spans - n_cold;
    }
    if (skip + s >= n_spans) return;
    s = order[skip + s];
    if (s >= n_spans) return;
  }
  const u32 c = threadIdx.x % LPR;
  const u32 b = s * span;
  if (b >= n) return;
  const u32 e = min(b + span, n);
  const bool col_ok = c * 4 < D;

  bool first_row_open = (b > 0) && (sr[b - 1] == sr[b]);  // the span starts inside a row begun earlier
  u32 flags = 0, started = 0;
  d4 acc = {0.0, 0.0, 0.0, 0.0};

  // LPR > PB: the group keeps a window of LPR consecutive list entries (lane c holds entry
  // window start + c, plus the first row id after the window) and refills it with three loads
  // every LPR occurrences, instead of two small loads per batch of PB
  u32 win_r = NO_ROW, win_g = 0u, win_next = NO_ROW;
  for (u32 i0 = b; i0 < e; i0 += PB) {
    u32 r[PB + 1], g[PB];
    if constexpr (LPR > PB && LPR % PB == 0) {
      const u32 o = (i0 - b) % LPR;
      if (o == 0) {
        win_r = (i0 + c < n) ? sr[i0 + c] : NO_ROW;
        win_g = (i0 + c < e) ? ss[i0 + c] : 0u;
        win_next = (i0 + LPR < n) ? sr[i0 + LPR] : NO_ROW;
      }
#pragma unroll
      for (int i = 0; i <= PB; ++i) {
        const u32 from_win = __shfl(win_r, (int)((o + i) % LPR), LPR);
        r[i] = (o + i < (u32)LPR) ? from_win : win_next;
      }
#pragma unroll
      for (int i = 0; i < PB; ++i) g[i] = __shfl(win_g, (int)(o + i), LPR);
    } else if constexpr (LPR > PB) {  // one coalesced index load per group, then broadcast
      const u32 mine_r = (c <= PB && i0 + c < n) ? sr[i0 + c] : NO_ROW;
      const u32 mine_g = (c < PB && i0 + c < e) ? ss[i0 + c] : 0u;
#pragma unroll
      for (int i = 0; i <= PB; ++i) r[i] = __shfl(mine_r, i, LPR);
#pragma unroll
      for (int i = 0; i < PB; ++i) g[i] = __shfl(mine_g, i, LPR);
    } else {
#pragma unroll
      for (int i = 0; i <= PB; ++i) r[i] = (i0 + i < n) ? sr[i0 + i] : NO_ROW;
#pragma unroll
      for (int i = 0; i < PB; ++i) g[i] = (i0 + i < e) ? ss[i0 + i] : 0u;
    }
    bool valid[PB], ends[PB], whole[PB];
    bool fo = first_row_open;
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      valid[i] = i0 + i < e;
      ends[i] = valid[i] && r[i + 1] != r[i];  // last occurrence of its row (r[i+1] is NO_ROW past the end)
      whole[i] = ends[i] && !fo;               // and the row began inside this span
      if (ends[i]) fo = false;
    }
    f4 gv[PB];
    RowState4 st[PB];
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      gv[i].x = gv[i].y = gv[i].z = gv[i].w = 0.0f;
      if (valid[i] && col_ok) {
        if constexpr (GB) {
          const uint2 raw = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(grad_any) + (u64)g[i] * D + 4 * c);
          gv[i].x = __uint_as_float(raw.x << 16);
          gv[i].y = __uint_as_float(raw.x & 0xFFFF0000u);
          gv[i].z = __uint_as_float(raw.y << 16);
          gv[i].w = __uint_as_float(raw.y & 0xFFFF0000u);
        } else {
#if CTR_PUSH_NT_GRAD
          gv[i] = ldg4_stream(static_cast<const float*>(grad_any) + (u64)g[i] * D + 4 * c);
#else
          gv[i] = ldg4(static_cast<const float*>(grad_any) + (u64)g[i] * D + 4 * c);
#endif
        }
      }
    }
#pragma unroll
    for (int i = 0; i < PB; ++i)
      if (whole[i] && col_ok) st[i] = load_row4<KIND>(values, vhat, r[i], D, rf, c);
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      if (valid[i]) {
        acc.x += (double)gv[i].x;
        acc.y += (double)gv[i].y;
        acc.z += (double)gv[i].z;
        acc.w += (double)gv[i].w;
        if (ends[i]) {
          if (whole[i]) {
            finish_row_loaded<KIND>(r[i], st[i], acc, c, col_ok, values, row_state, D, rf, P);
            ++started;
          } else {  // end of the row that was open on entry
            if (col_ok) store_partial(head_part, s, D, c, acc);
            flags |= SF_HEAD;
            first_row_open = false;
          }
          acc.x = acc.y = acc.z = acc.w = 0.0;
        }
      }
    }
  }

  // the last occurrence did not end its row: the row goes on in the next span
  if (sr[e - 1] == ((e < n) ? sr[e] : NO_ROW)) {
    if (first_row_open) {  // the whole span lies inside one row that began earlier
      if (col_ok) store_partial(head_part, s, D, c, acc);
      flags |= SF_HEAD;
    } else {
      if (col_ok) store_partial(tail_part, s, D, c, acc);
      flags |= SF_TAIL;
      ++started;
    }
  }
  if (c == 0) {
    span_flags[s] = (sr[b] << 2) | flags;  // first row id of the span above the two flag bits
    span_rows[s] = started;                // rows that START in this span
  }
}

#define CTR_PUSH_SPAN_ARGS                                                                                      \
  const DevHeader *hdr, const u32 *__restrict__ sr, const u32 *__restrict__ ss, u32 n, u32 span,               \
      const void *__restrict__ grad, float *__restrict__ values, const float *__restrict__ vhat,               \
      u32 *__restrict__ row_state, u32 D, u32 rf, AdamParams P, double *__restrict__ head_part,                \
      double *__restrict__ tail_part, u32 *__restrict__ span_flags, u32 *__restrict__ span_rows,               \
      const u32 *__restrict__ order, const u32 *__restrict__ cold_count
#define CTR_PUSH_SPAN_PASS                                                                                      \
  hdr, sr, ss, n, span, grad, values, vhat, row_state, D, rf, P, head_part, tail_part, span_flags, span_rows, \
      order, cold_count

// one kernel per step kind (the dispatch macro on the host takes kernels templated on LPR only)
#define CTR_DEFINE_PUSH_SPAN(NAME, KIND)                                                          \
  template <int LPR>                                                                              \
  __global__ void __launch_bounds__(BLOCK, CTR_PUSH_MIN_WAVES) NAME(CTR_PUSH_SPAN_ARGS) {         \
    push_span_body<LPR, KIND, false>(CTR_PUSH_SPAN_PASS);                                         \
  }                                                                                               \
  template <int LPR>                                                                              \
  __global__ void __launch_bounds__(BLOCK, CTR_PUSH_MIN_WAVES) NAME##_g16(CTR_PUSH_SPAN_ARGS) {   \
    push_span_body<LPR, KIND, true>(CTR_PUSH_SPAN_PASS);                                          \
  }
#define CTR_PUSH_HOT_ARGS                                                                                       \
  const DevHeader *hdr, const u32 *__restrict__ sr, const u32 *__restrict__ ss, u32 n, u32 span,               \
      const void *__restrict__ grad, u32 D, double *__restrict__ head_part, double *__restrict__ tail_part,    \
      u32 *__restrict__ span_flags, u32 *__restrict__ span_rows, const u32 *__restrict__ order,                \
      const u32 *__restrict__ cold_count
template <int LPR>
__global__ void __launch_bounds__(BLOCK) k_push_hot(CTR_PUSH_HOT_ARGS) {
  push_hot_body<LPR, false>(hdr, sr, ss, n, span, grad, D, head_part, tail_part, span_flags, span_rows, order,
                            cold_count);
}
template <int LPR>
__global__ void __launch_bounds__(BLOCK) k_push_hot_g16(CTR_PUSH_HOT_ARGS) {
  push_hot_body<LPR, true>(hdr, sr, ss, n, span, grad, D, head_part, tail_part, span_flags, span_rows, order,
                           cold_count);
}

CTR_DEFINE_PUSH_SPAN(k_push_span, STEP_ADAM_OWN)
CTR_DEFINE_PUSH_SPAN(k_push_span_shared, STEP_ADAM_SHARED)
CTR_DEFINE_PUSH_SPAN(k_push_span_adagrad, STEP_ADAGRAD)
CTR_DEFINE_PUSH_SPAN(k_push_span_kingma, STEP_ADAM_KINGMA)

// Number of leading lanes (from lane 0) whose predicate holds; wave-uniform.
__device__ __forceinline__ u32 leading_true(bool pred) {
  const u64 inv = ~__ballot(pred);
  return inv ? (u32)(__ffsll((long long)inv) - 1) : 64u;
}

// Combines per-group binary64 partial sums of a wave (groups of LPR lanes, same column layout).
template <int LPR>
__device__ __forceinline__ void combine_groups(d4& a) {
#pragma unroll
  for (int off = LPR; off < WAVE; off <<= 1) {
    a.x += __shfl_xor(a.x, off, WAVE);
    a.y += __shfl_xor(a.y, off, WAVE);
    a.z += __shfl_xor(a.z, off, WAVE);
    a.w += __shfl_xor(a.w, off, WAVE);
  }
}

// One wave per block of SPANS_PER_BLOCK spans (block j >= 1): sums the heads of the
// block's leading spans that continue the row open at the block's start.
template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_push_block_heads(const DevHeader* hdr, const u32* __restrict__ sr, u32 n_spans, u32 span, u32 D,
                   const double* __restrict__ head_part, double* __restrict__ block_head,
                   const u32* __restrict__ span_flags) {
  if (hdr->status) return;
  constexpr int GPW = WAVE / LPR;
  const u32 j = (blockIdx.x * BLOCK + threadIdx.x) / WAVE;  // wave-uniform
  const u32 first = j * SPANS_PER_BLOCK;
  if (j == 0 || first >= n_spans) return;
  const int lane = lane_id();
  const u32 c = lane % LPR, grp = lane / LPR;
  const bool col_ok = c * 4 < D;
  const u32 row = sr[first * span - 1];
  const u32 t = first + lane;
  const u32 n_lead = leading_true(t < n_spans && (span_flags[t] >> 2) == row);  // coalesced, unlike sr[t * span]
  if (n_lead == 0) return;
  d4 acc = {0.0, 0.0, 0.0, 0.0};
  if (col_ok)
    for (u32 k = grp; k < n_lead; k += GPW) add_partial(head_part, first + k, D, c, acc);
  combine_groups<LPR>(acc);
  if (grp == 0 && col_ok) store_partial(block_head, j, D, c, acc);
}

// One wave per span that holds a tail: tail + heads of the following spans of
// the same block + block sums of the following blocks, while they continue
// the same row; then the row update.
template <int LPR, int KIND>
__device__ __forceinline__ void push_fixup_body(const DevHeader* hdr, const u32* __restrict__ sr, u32 n, u32 n_spans,
                                                u32 span, float* __restrict__ values,
                                                const float* __restrict__ vhat, u32* __restrict__ row_state, u32 D,
                                                u32 rf, const AdamParams& P_in, const double* __restrict__ head_part,
                                                const double* __restrict__ tail_part,
                                                const double* __restrict__ block_head,
                                                const u32* __restrict__ span_flags) {
  if (hdr->status) return;
  AdamParams P = P_in;
  if constexpr (KIND == STEP_ADAM_KINGMA) {
    P.bc1 = hdr->bc1;
    P.bc2 = hdr->bc2;
  }
  constexpr int GPW = WAVE / LPR;
  const u32 s = (blockIdx.x * BLOCK + threadIdx.x) / WAVE;  // wave-uniform
  if (s >= n_spans) return;
  if (!(span_flags[s] & SF_TAIL)) return;
  const int lane = lane_id();
  const u32 c = lane % LPR, grp = lane / LPR;
  const bool col_ok = c * 4 < D;
  const u32 row = sr[(s + 1) * span - 1];  // a tail means the span is full and the list goes on
  const u32 n_blocks = (n_spans + SPANS_PER_BLOCK - 1) / SPANS_PER_BLOCK;
  const u32 blk_end = min((s / SPANS_PER_BLOCK + 1) * SPANS_PER_BLOCK, n_spans);

  d4 acc = {0.0, 0.0, 0.0, 0.0};
  RowState4 st;
  if (grp == 0 && col_ok) {
    add_partial(tail_part, s, D, c, acc);
    st = load_row4<KIND>(values, vhat, row, D, rf, c);
  }
  // spans after s inside its block (at most SPANS_PER_BLOCK - 1 = one per lane)
  const u32 t = s + 1 + lane;
  const u32 n_in = leading_true(t < blk_end && (span_flags[t] >> 2) == row);
  if (col_ok)
    for (u32 k = grp; k < n_in; k += GPW) add_partial(head_part, s + 1 + k, D, c, acc);
  if (s + 1 + n_in == blk_end) {  // the row reaches the end of the block: go on block by block
    for (u32 jb = s / SPANS_PER_BLOCK + 1; jb < n_blocks; jb += WAVE) {
      const u32 jj = jb + lane;
      const u32 nb = leading_true(jj < n_blocks && (span_flags[jj * SPANS_PER_BLOCK] >> 2) == row);
      if (col_ok)
        for (u32 k = grp; k < nb; k += GPW) add_partial(block_head, jb + k, D, c, acc);
      if (nb < WAVE) break;
    }
  }
  combine_groups<LPR>(acc);
  if (grp == 0) finish_row_loaded<KIND>(row, st, acc, c, col_ok, values, row_state, D, rf, P);
}

#define CTR_PUSH_FIXUP_ARGS                                                                                     \
  const DevHeader *hdr, const u32 *__restrict__ sr, u32 n, u32 n_spans, u32 span, float *__restrict__ values,  \
      const float *__restrict__ vhat, u32 *__restrict__ row_state, u32 D, u32 rf, AdamParams P,                \
      const double *__restrict__ head_part, const double *__restrict__ tail_part,                              \
      const double *__restrict__ block_head, const u32 *__restrict__ span_flags
#define CTR_PUSH_FIXUP_PASS \
  hdr, sr, n, n_spans, span, values, vhat, row_state, D, rf, P, head_part, tail_part, block_head, span_flags

#define CTR_DEFINE_PUSH_FIXUP(NAME, KIND)                                    \
  template <int LPR>                                                         \
  __global__ void __launch_bounds__(BLOCK) NAME(CTR_PUSH_FIXUP_ARGS) {       \
    push_fixup_body<LPR, KIND>(CTR_PUSH_FIXUP_PASS);                         \
  }
CTR_DEFINE_PUSH_FIXUP(k_push_fixup, STEP_ADAM_OWN)
CTR_DEFINE_PUSH_FIXUP(k_push_fixup_shared, STEP_ADAM_SHARED)
CTR_DEFINE_PUSH_FIXUP(k_push_fixup_adagrad, STEP_ADAGRAD)
CTR_DEFINE_PUSH_FIXUP(k_push_fixup_kingma, STEP_ADAM_KINGMA)

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

// k-step merge.  One group of LPR lanes per row in use; rows nobody touched since the last merge
// are skipped.  Sums in binary64, rounded once.
//   PROSE == false (Algorithm 2 as printed): shared v = mean_j v_j; every replica's x becomes
//     mean_j (x_j - [pending_j] lr m_j / sqrt(shared v)); local v_j stay.
//   PROSE == true (Section 4's prose: standard Adam locally, weights and v averaged): every
//     replica's x becomes mean_j x_j and every v_j becomes mean_j v_j.
template <int LPR, bool PROSE>
__device__ __forceinline__ void merge_body(DevHeader* hdr, float* __restrict__ values, u64 replica_stride,
                                           u32 W, float* __restrict__ vhat, u32* __restrict__ row_state, u32 D,
                                           float lr) {
  if (hdr->status) return;
  const u32 n_rows = hdr->n_rows;
  const u32 c = threadIdx.x % LPR;
  const u32 groups = gridDim.x * (BLOCK / LPR);
  const bool col_ok = c * 4 < D;
  u32 merged = 0, pend = 0;
  for (u32 row = (blockIdx.x * BLOCK + threadIdx.x) / LPR; row < n_rows; row += groups) {
    const u32 st = row_state[row];
    if (!(st & RS_TOUCHED)) continue;
    if (col_ok) {
      // replicas are taken eight at a time: the eight loads of a batch are independent of each other
      // and issued together; the sums run over the replicas in ascending order whatever the batching
      constexpr int MB = CTR_MERGE_MB;
      float* base = values + (u64)row * 3 * D + 4 * c;
      d4 vs = {0.0, 0.0, 0.0, 0.0};
      for (u32 j0 = 0; j0 < W; j0 += MB) {
        f4 vv[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i)
          if (j0 + i < W) vv[i] = ldg4(base + (u64)(j0 + i) * replica_stride + 2 * D);
#pragma unroll
        for (int i = 0; i < MB; ++i)
          if (j0 + i < W) {
            vs.x += (double)vv[i].x; vs.y += (double)vv[i].y; vs.z += (double)vv[i].z; vs.w += (double)vv[i].w;
          }
      }
      const double w = (double)W;
      f4 vh;
      vh.x = (float)(vs.x / w); vh.y = (float)(vs.y / w); vh.z = (float)(vs.z / w); vh.w = (float)(vs.w / w);
      d4 rs = {0.0, 0.0, 0.0, 0.0};
      if constexpr (PROSE) {
        for (u32 j = 0; j < W; ++j) stg4(base + j * replica_stride + 2 * D, vh);
      } else {
        stg4(vhat + (u64)row * D + 4 * c, vh);
        rs = d4{rsqrt_refined(vh.x), rsqrt_refined(vh.y), rsqrt_refined(vh.z), rsqrt_refined(vh.w)};
      }
      const double lrd = (double)lr;
      d4 xs = {0.0, 0.0, 0.0, 0.0};
      for (u32 j0 = 0; j0 < W; j0 += MB) {
        f4 xx[MB], mm[MB];
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          mm[i] = f4{0.0f, 0.0f, 0.0f, 0.0f};
          if (j0 + i < W) {
            xx[i] = ldg4(base + (u64)(j0 + i) * replica_stride);
            if (!PROSE && (st & (1u << (j0 + i)))) mm[i] = ldg4(base + (u64)(j0 + i) * replica_stride + D);
          }
        }
#pragma unroll
        for (int i = 0; i < MB; ++i)
          if (j0 + i < W) {
            d4 y = {(double)xx[i].x, (double)xx[i].y, (double)xx[i].z, (double)xx[i].w};
            if (!PROSE && (st & (1u << (j0 + i)))) {
              y.x -= lrd * (double)mm[i].x * rs.x;
              y.y -= lrd * (double)mm[i].y * rs.y;
              y.z -= lrd * (double)mm[i].z * rs.z;
              y.w -= lrd * (double)mm[i].w * rs.w;
            }
            xs.x += y.x; xs.y += y.y; xs.z += y.z; xs.w += y.w;
          }
      }
      f4 xb;
      xb.x = (float)(xs.x / w); xb.y = (float)(xs.y / w); xb.z = (float)(xs.z / w); xb.w = (float)(xs.w / w);
      for (u32 j = 0; j < W; ++j) stg4(base + j * replica_stride, xb);
    }
    if (c == 0) {
      row_state[row] = 0;
      ++merged;
      if (!PROSE) pend += (u32)__popc(st & ~RS_TOUCHED);
    }
  }
  // rows averaged (and deferred steps applied) by this launch, for the byte accounting of the merge:
  // one atomic per wave and counter
  for (int off = WAVE / 2; off > 0; off >>= 1) {
    merged += __shfl_xor(merged, off, WAVE);
    pend += __shfl_xor(pend, off, WAVE);
  }
  if (lane_id() == 0 && merged) {
    atomicAdd(&hdr->rows_merged, (u64)merged);
    if (pend) atomicAdd(&hdr->merge_pending, (u64)pend);
  }
}

template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_merge(DevHeader* hdr, float* __restrict__ values, u64 replica_stride, u32 W, float* __restrict__ vhat,
        u32* __restrict__ row_state, u32 D, float lr) {
  merge_body<LPR, false>(hdr, values, replica_stride, W, vhat, row_state, D, lr);
}
template <int LPR>
__global__ void __launch_bounds__(BLOCK)
k_merge_prose(DevHeader* hdr, float* __restrict__ values, u64 replica_stride, u32 W,
              float* __restrict__ vhat, u32* __restrict__ row_state, u32 D, float lr) {
  merge_body<LPR, true>(hdr, values, replica_stride, W, vhat, row_state, D, lr);
}

// Measurement aid: a plain streaming copy (16 bytes per lane and access, grid-stride), the practical
// ceiling of this GPU's memory system against which the kernels above are also reported.
// n16 = number of 16-byte units.  STREAM: use the non-temporal hint on both sides.
template <bool STREAM>
__global__ void __launch_bounds__(BLOCK) k_stream_copy(const vf4* __restrict__ src, vf4* __restrict__ dst, u64 n16) {
  const u64 stride = (u64)gridDim.x * BLOCK;
  u64 i = (u64)blockIdx.x * BLOCK + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    vf4 a, b, c, d;
    if constexpr (STREAM) {
      a = __builtin_nontemporal_load(src + i);
      b = __builtin_nontemporal_load(src + i + stride);
      c = __builtin_nontemporal_load(src + i + 2 * stride);
      d = __builtin_nontemporal_load(src + i + 3 * stride);
      __builtin_nontemporal_store(a, dst + i);
      __builtin_nontemporal_store(b, dst + i + stride);
      __builtin_nontemporal_store(c, dst + i + 2 * stride);
      __builtin_nontemporal_store(d, dst + i + 3 * stride);
    } else {
      a = src[i]; b = src[i + stride]; c = src[i + 2 * stride]; d = src[i + 3 * stride];
      dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace ctr
