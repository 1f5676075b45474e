// bf16 x bf16 -> fp32 matrix product on the gfx950 matrix cores, hand-written for the dense tower.
//
// Paper: Algorithm 1's train_mini-batch step on the network of Section 2.1 - the three products of
// a fully connected layer (forward Z = H W, weight gradient dW = H^T dZ, input gradient
// dH = dZ W^T).  They are the only dense contractions of the training step.
//
// C[M x N] (row-major, N contiguous) = A[M x K] B[K x N].  Either operand may be stored with the
// contraction index contiguous ("k-contiguous": A as M rows of K, B as N rows of K) or with its
// other index contiguous (A as K rows of M, B as K rows of N); the three products of a row-major
// layer need three of the four combinations, and none of them needs a transposed copy in memory.
//
// One workgroup of 4 waves (2 x 2) computes a 256 x 256 tile of C: each wave holds a 128 x 128
// sub-tile as 4 x 4 accumulators of v_mfma_f32_32x32x16_bf16 (256 accumulator registers per lane).
// The contraction runs in steps of 64: the two operand tiles (256 x 64 each) are fetched from
// memory into registers one step ahead (8 loads of 16 bytes per lane and operand), written to one of
// two LDS buffers as rows of 64 k-contiguous values (128 bytes), and read back as the 16-byte
// fragments the matrix instruction takes.  An operand whose memory layout is not k-contiguous is
// transposed on the way, in registers: a lane fetches an 8 x 8 block as 8 vectors along the
// contiguous index and turns it into 8 vectors along k with 32 byte-permute instructions.
// The 16-byte chunks of an LDS row are XOR-swizzled with the row number, so that the 8 lanes the
// LDS serves together always fall on 8 different chunks, for the writes of both layouts and for
// the fragment reads.
// A long contraction with few output tiles (the weight gradients) is split along K over several
// workgroups; each writes its fp32 partial tile, and a second launch adds the partials in a fixed
// order and applies the epilogue, so results do not depend on scheduling.
// All dimensions are multiples of 8 (16-byte vectors never straddle an edge); tiles that stick out
// of the matrices are zero-filled on load and clipped on store.
#pragma once
#include "common.h"

namespace ctr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes in flight between memory, registers and LDS

constexpr u32 GEMM_BM = 256, GEMM_BN = 256, GEMM_BK = 64;
constexpr u32 GEMM_TILE_BYTES = GEMM_BM * GEMM_BK * 2;  // one operand tile in LDS: 32 KB
constexpr u32 GEMM_LDS_BYTES = 4 * GEMM_TILE_BYTES;     // A and B, two buffers each: 128 KB
constexpr u32 GEMM_GROUP_M = 8;                         // tile rows walked together (operand reuse in L2)

// what happens to a finished element of C
enum GemmEpilogue : int {
  EPI_F32 = 0,             // C32[m, n] = acc
  EPI_BIAS_RELU_BF16 = 1,  // C16[m, n] = bf16(max(acc + bias[n], 0))       (forward: the next activation)
  EPI_BF16 = 2,            // C16[m, n] = bf16(acc)
  EPI_RELU_MASK_BF16 = 3,  // C16[m, n] = bf16(mask[m, n] > 0 ? acc : 0)    (input gradient through a ReLU)
  EPI_PARTIAL = 4          // internal: partial[split][m][n] = acc (a split contraction)
};

struct GemmArgs {
  const bf16_t* A;
  const bf16_t* B;
  u32 lda, ldb;  // elements between consecutive rows of the operand as stored
  u32 M, N, K;
  u32 n_split, k_per_split;  // K is cut into n_split ranges of k_per_split (a multiple of GEMM_BK)
  u32 tiles_m, tiles_n;
  float* C32;
  bf16_t* C16;
  u32 ldc;
  const float* bias;   // EPI_BIAS_RELU_BF16
  const bf16_t* mask;  // EPI_RELU_MASK_BF16, laid out like C
  float* partial;      // n_split > 1: [n_split][M][N] fp32
  int epilogue;
};

// Epilogue on 4 consecutive columns of one row (n a multiple of 4; C, mask and partial rows are 16-byte
// aligned because every dimension is a multiple of 8).
__device__ __forceinline__ void gemm_emit4(const GemmArgs& g, int epilogue, u32 m, u32 n, f4 v, u32 split) {
  if (epilogue == EPI_PARTIAL) {
    stg4(g.partial + ((u64)split * g.M + m) * g.N + n, v);
    return;
  }
  const u64 i = (u64)m * g.ldc + n;
  if (epilogue == EPI_F32) {
    stg4(g.C32 + i, v);
  } else if (epilogue == EPI_BIAS_RELU_BF16) {
    const f4 b = ldg4(g.bias + n);
    stg4_bf16(g.C16 + i, f4{fmaxf(v.x + b.x, 0.0f), fmaxf(v.y + b.y, 0.0f), fmaxf(v.z + b.z, 0.0f), fmaxf(v.w + b.w, 0.0f)});
  } else if (epilogue == EPI_BF16) {
    stg4_bf16(g.C16 + i, v);
  } else {
    const ushort4 a = *reinterpret_cast<const ushort4*>(g.mask + i);
    stg4_bf16(g.C16 + i, f4{from_bf16(a.x) > 0.0f ? v.x : 0.0f, from_bf16(a.y) > 0.0f ? v.y : 0.0f,
                             from_bf16(a.z) > 0.0f ? v.z : 0.0f, from_bf16(a.w) > 0.0f ? v.w : 0.0f});
  }
}

// A wave's 128 x 128 accumulators to memory, through LDS: in two passes of 64 rows the wave writes its
// accumulators to its own quarter of the (now free) operand buffers in the matrix instruction's layout
// (register r of a lane is row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32 of a 32 x 32 block)
// and reads them back as rows, so that every lane stores 4 consecutive columns (16 bytes of fp32) and a
// wave-wide store covers two rows of 512 contiguous bytes; the epilogue is applied on the way.  The
// read-back is a loop, which keeps the code short.  All waves of the workgroup take the barriers.
__device__ __forceinline__ void gemm_write_tile(const GemmArgs& g, int epilogue, const f32x16 (&acc)[4][4], char* lds,
                                                u32 m_wave, u32 n_wave, u32 split) {
  const u32 lane = (u32)lane_id();
  float* region = reinterpret_cast<float*>(lds + (u32)wave_id() * (GEMM_LDS_BYTES / 4));
  const u32 frag_row = lane & 31u, frag_half = lane >> 5;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();  // the buffers are free: operand reads (pass 0) or the previous pass's read-back are done
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          region[(h * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4)) * 128 + ni * 32 + frag_row] = acc[2 * pass + h][ni][r];
    __syncthreads();
    const u32 n = n_wave + (lane & 31u) * 4;
    for (u32 it = 0; it < 32; ++it) {
      const u32 row = it * 2 + (lane >> 5);
      const u32 m = m_wave + pass * 64 + row;
      const f4 v = *reinterpret_cast<const f4*>(region + row * 128 + (lane & 31u) * 4);
      if (m < g.M && n < g.N) gemm_emit4(g, epilogue, m, n, v, split);
    }
  }
}

// 8 x 8 transpose of 16-bit values held as 8 vectors of 8: T[i] element k = R[k] element i.
__device__ __forceinline__ void gemm_transpose8x8(const u32x4 (&R)[8], u32x4 (&T)[8]) {
  u32 r[8][4], t[8][4];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    r[j][0] = R[j].x; r[j][1] = R[j].y; r[j][2] = R[j].z; r[j][3] = R[j].w;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      // bytes 0..3 of the selector address the second source, 4..7 the first
      t[2 * q][p] = __builtin_amdgcn_perm(r[2 * p + 1][q], r[2 * p][q], 0x05040100u);      // low halves
      t[2 * q + 1][p] = __builtin_amdgcn_perm(r[2 * p + 1][q], r[2 * p][q], 0x07060302u);  // high halves
    }
#pragma unroll
  for (int i = 0; i < 8; ++i) T[i] = u32x4{t[i][0], t[i][1], t[i][2], t[i][3]};
}

// Where this lane's 8 vectors of an operand tile lie, as byte offsets from a base that is the same for
// the whole workgroup and moves along k from step to step (so the base lives in scalar registers and
// only these 8 offsets in vector registers).  Rows beyond the matrix are redirected to row 0 (always
// readable): they only feed elements of C that are never stored.  Offsets are 32 bits: an operand
// holds less than 4 GiB.
// KC: the operand is stored as rows of k (element (row, k) at P[row * ld + k]): vector j is row
// rb + 32 j, k = 8 kb .. 8 kb + 7.  Otherwise it is stored as rows of the other index (element
// (row, k) at P[k * ld + row]): vector r is k = 8 kb + r, rows 8 rb .. 8 rb + 7.
template <bool KC>
__device__ __forceinline__ void gemm_offsets(u32 ld, u32 rows_total, u32 row0, u32 (&off)[8]) {
  const u32 kb = threadIdx.x & 7u, rb = threadIdx.x >> 3;
  if constexpr (KC) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32 row = row0 + rb + 32 * j;
      off[j] = ((row < rows_total ? row : 0u) * ld + kb * 8) * 2u;
    }
  } else {
    const u32 row = row0 + rb * 8;
#pragma unroll
    for (int r = 0; r < 8; ++r) off[r] = ((kb * 8 + r) * ld + (row < rows_total ? row : 0u)) * 2u;
  }
}

// The 8 loads of one operand tile at k0, for a tile that lies inside K (k0 + 64 <= K).  Nothing here
// depends on loaded data, so the loads stay in flight while earlier tiles are multiplied.
template <bool KC>
__device__ __forceinline__ void gemm_fetch(const bf16_t* __restrict__ P, u32 ld, u32 k0, const u32 (&off)[8],
                                           u32x4 (&R)[8]) {
  const char* base = reinterpret_cast<const char*>(P) + (KC ? (u64)k0 * 2u : (u64)k0 * ld * 2u);
#pragma unroll
  for (int j = 0; j < 8; ++j) R[j] = *reinterpret_cast<const u32x4*>(base + off[j]);
}

// The same for a tile that reaches beyond K (the last step of a contraction whose length is no multiple
// of 64, or a step requested ahead beyond the end): vectors at k >= K are fetched from the operand's
// first bytes instead (always readable); gemm_stage replaces them by zeros.
template <bool KC>
__device__ __forceinline__ void gemm_fetch_tail(const bf16_t* __restrict__ P, u32 ld, u32 K, u32 k0,
                                                const u32 (&off)[8], u32x4 (&R)[8]) {
  const u32 kb = threadIdx.x & 7u;
  const char* first = reinterpret_cast<const char*>(P);
  const char* base = first + (KC ? (u64)k0 * 2u : (u64)k0 * ld * 2u);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const bool in = KC ? (k0 + kb * 8 < K) : (k0 + kb * 8 + (u32)j < K);
    R[j] = *reinterpret_cast<const u32x4*>(in ? base + off[j] : first);
  }
}

// ... and from the registers into an LDS tile: row r holds its 64 k-values as 8 chunks of 16 bytes,
// chunk c stored at position c ^ (r & 7).  k_tail: the tile reaches beyond K (k0 + 64 > K), so the
// vectors with k >= K are replaced by zeros first.
template <bool KC>
__device__ __forceinline__ void gemm_stage(char* lds, u32x4 (&R)[8], bool k_tail, u32 K, u32 k0) {
  const u32 kb = threadIdx.x & 7u, rb = threadIdx.x >> 3;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (k_tail) {  // uniform over the workgroup, taken at most once per work item
    if constexpr (KC) {
      if (k0 + kb * 8 >= K) {
#pragma unroll
        for (int j = 0; j < 8; ++j) R[j] = zero;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 8; ++r)
        if (k0 + kb * 8 + r >= K) R[r] = zero;
    }
  }
  if constexpr (KC) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const u32 row = rb + 32 * j;
      *reinterpret_cast<u32x4*>(lds + row * 128 + ((kb ^ (row & 7u)) << 4)) = R[j];
    }
  } else {
    u32x4 T[8];
    gemm_transpose8x8(R, T);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u32 row = rb * 8 + i;
      *reinterpret_cast<u32x4*>(lds + row * 128 + ((kb ^ (u32)i) << 4)) = T[i];
    }
  }
}

// One contraction step of a wave: 4 sub-steps of 16, each 4 + 4 fragment reads from LDS and 4 x 4 matrix
// instructions.  The fragments of sub-step kk + 1 are read while the products of sub-step kk run, and
// (FETCH) the 16 global loads of the next step's tiles are spread over the step, one per four matrix
// instructions; the scheduling directives at the end pin that interleaving (without them the compiler
// gathers the loads at the start and the LDS reads right before their first use).
template <bool A_KC, bool B_KC, bool FETCH>
__device__ __forceinline__ void gemm_step(const char* la, const char* lb, u32 frag_half, u32 frag_swz,
                                          f32x16 (&acc)[4][4], const bf16_t* __restrict__ Ap,
                                          const bf16_t* __restrict__ Bp, const GemmArgs& g, const u32 (&offa)[8],
                                          const u32 (&offb)[8], u32 k_a, u32 k_b, u32x4 (&ra)[8], u32x4 (&rb)[8]) {
  if constexpr (FETCH) {
    gemm_fetch<A_KC>(Ap, g.lda, k_a, offa, ra);
    gemm_fetch<B_KC>(Bp, g.ldb, k_b, offb, rb);
  }
  bf16x8 a[2][4], b[2][4];
  {
    const u32 chunk = (frag_half ^ frag_swz) << 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[0][i] = *reinterpret_cast<const bf16x8*>(la + i * 32 * 128 + chunk);
      b[0][i] = *reinterpret_cast<const bf16x8*>(lb + i * 32 * 128 + chunk);
    }
  }
#pragma unroll
  for (u32 kk = 0; kk < GEMM_BK / 16; ++kk) {
    const u32 cur = kk & 1u, nxt = cur ^ 1u;
    if (kk + 1 < GEMM_BK / 16) {
      const u32 chunk = ((2 * (kk + 1) + frag_half) ^ frag_swz) << 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[nxt][i] = *reinterpret_cast<const bf16x8*>(la + i * 32 * 128 + chunk);
        b[nxt][i] = *reinterpret_cast<const bf16x8*>(lb + i * 32 * 128 + chunk);
      }
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][mi], b[cur][ni], acc[mi][ni], 0, 0, 0);
  }
  // instruction classes: 0x008 matrix, 0x020 memory read, 0x100 LDS read
  __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);  // fragments of sub-step 0
#pragma unroll
  for (int kk = 0; kk < 3; ++kk)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (FETCH && kk < 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (FETCH && kk < 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
  __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
}

// The operand pointers are kernel parameters of their own (not members of the argument block), so that
// the compiler knows them to be global memory.
// EARLY: the registers are refilled with the next tiles as soon as they have been staged (before the
// barrier, all 16 loads at once) instead of during the first half of the following step.  Long
// contractions gain from it (the requests get the barrier and the fragment reads as extra time), short
// ones lose (measured: 300 and 64 steps per work item -5 % and -2 %, 16 steps +10 %); the host picks.
template <bool A_KC, bool B_KC, bool EARLY>
__global__ void __launch_bounds__(256, 1)
k_gemm_bf16(const bf16_t* __restrict__ Ap, const bf16_t* __restrict__ Bp, GemmArgs g) {
  extern __shared__ __align__(16) char gemm_lds[];
  // work item -> (split, tile row, tile column).  Workgroups are dealt to the 8 XCDs round-robin: ids
  // are re-numbered so that one XCD gets a contiguous range, and tile rows are walked in groups so
  // that the tiles an L2 sees at about the same time share their operand panels.
  const u32 tiles = g.tiles_m * g.tiles_n, total = tiles * g.n_split;
  u32 id = blockIdx.x;
  if (total % 8u == 0u) id = (blockIdx.x % 8u) * (total / 8u) + blockIdx.x / 8u;
  const u32 split = id / tiles, tid = id % tiles;
  const u32 group_size = GEMM_GROUP_M * g.tiles_n;
  const u32 first_m = (tid / group_size) * GEMM_GROUP_M;
  const u32 gm = min(GEMM_GROUP_M, g.tiles_m - first_m);
  const u32 tm = first_m + (tid % group_size) % gm, tn = (tid % group_size) / gm;
  const u32 m0 = tm * GEMM_BM, n0 = tn * GEMM_BN;
  const u32 k_begin = split * g.k_per_split, k_end = min(g.K, k_begin + g.k_per_split);
  const u32 n_steps = (k_end - k_begin + GEMM_BK - 1) / GEMM_BK;

  const int lane = lane_id(), w = wave_id();
  const u32 wm = (u32)w >> 1, wn = (u32)w & 1u;
  // fragment addressing: lane reads row (lane & 31) of a 32-row block, chunk 2 * kk + (lane >> 5)
  const u32 frag_row = (u32)lane & 31u, frag_half = (u32)lane >> 5, frag_swz = (u32)lane & 7u;
  const u32 a_base = (wm * 128 + frag_row) * 128, b_base = (wn * 128 + frag_row) * 128;

  f32x16 acc[4][4];
  {
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = zero;
  }

  // Operand tiles travel from memory to LDS through registers: while step s is multiplied, the tiles of
  // step s + 1 are requested (the 16 loads of a lane spread over the first half of the step) and, once the
  // products are issued, staged into the other LDS buffer.  One barrier per step: the buffer written was
  // last read before the previous barrier, the buffer read is next written after this one.
  // (Two register sets, i.e. requests two steps ahead, do not fit beside the 256 accumulator registers
  // and the fragments: the compiler spills inside the loop.)
  u32 offa[8], offb[8];
  gemm_offsets<A_KC>(g.lda, g.M, m0, offa);
  gemm_offsets<B_KC>(g.ldb, g.N, n0, offb);
  u32x4 ra[8], rb[8];
  if (n_steps > 0) {
    gemm_fetch_tail<A_KC>(Ap, g.lda, g.K, k_begin, offa, ra);
    gemm_fetch_tail<B_KC>(Bp, g.ldb, g.K, k_begin, offb, rb);
    const bool tail = k_begin + GEMM_BK > g.K;
    gemm_stage<A_KC>(gemm_lds, ra, tail, g.K, k_begin);
    gemm_stage<B_KC>(gemm_lds + 2 * GEMM_TILE_BYTES, rb, tail, g.K, k_begin);
  }
  __syncthreads();

  // the loop body exists once, with the fast fetch inside: a last step that reaches beyond K (a
  // contraction length that is no multiple of 64) is taken out of the loop
  const bool last_partial = n_steps > 0 && k_begin + n_steps * GEMM_BK > g.K;
  const u32 n_loop = n_steps - (last_partial ? 1u : 0u);  // steps whose tiles lie inside K
  u32 s = 0;
  if constexpr (EARLY) {
    if (n_loop > 1) {
      gemm_fetch<A_KC>(Ap, g.lda, k_begin + GEMM_BK, offa, ra);
      gemm_fetch<B_KC>(Bp, g.ldb, k_begin + GEMM_BK, offb, rb);
    }
    for (; s + 1 < n_loop; ++s) {
      const u32 buf = s & 1u;
      const u32 k_next = k_begin + (s + 1) * GEMM_BK;
      gemm_step<A_KC, B_KC, false>(gemm_lds + buf * GEMM_TILE_BYTES + a_base,
                                   gemm_lds + (2 + buf) * GEMM_TILE_BYTES + b_base, frag_half, frag_swz, acc, Ap, Bp, g,
                                   offa, offb, 0u, 0u, ra, rb);
      gemm_stage<A_KC>(gemm_lds + (buf ^ 1u) * GEMM_TILE_BYTES, ra, false, g.K, k_next);
      gemm_stage<B_KC>(gemm_lds + (2 + (buf ^ 1u)) * GEMM_TILE_BYTES, rb, false, g.K, k_next);
      if (s + 2 < n_loop) {
        gemm_fetch<A_KC>(Ap, g.lda, k_next + GEMM_BK, offa, ra);
        gemm_fetch<B_KC>(Bp, g.ldb, k_next + GEMM_BK, offb, rb);
      }
      __syncthreads();
    }
  } else {
    for (; s + 1 < n_loop; ++s) {
      const u32 buf = s & 1u;
      const u32 k_next = k_begin + (s + 1) * GEMM_BK;
      gemm_step<A_KC, B_KC, true>(gemm_lds + buf * GEMM_TILE_BYTES + a_base,
                                  gemm_lds + (2 + buf) * GEMM_TILE_BYTES + b_base, frag_half, frag_swz, acc, Ap, Bp, g,
                                  offa, offb, k_next, k_next, ra, rb);
      gemm_stage<A_KC>(gemm_lds + (buf ^ 1u) * GEMM_TILE_BYTES, ra, false, g.K, k_next);
      gemm_stage<B_KC>(gemm_lds + (2 + (buf ^ 1u)) * GEMM_TILE_BYTES, rb, false, g.K, k_next);
      __syncthreads();
    }
  }
  if (last_partial && n_steps > 1) {  // step s = n_steps - 2 with the partial tile behind it
    const u32 buf = s & 1u;
    const u32 k_next = k_begin + (s + 1) * GEMM_BK;
    gemm_fetch_tail<A_KC>(Ap, g.lda, g.K, k_next, offa, ra);
    gemm_fetch_tail<B_KC>(Bp, g.ldb, g.K, k_next, offb, rb);
    gemm_step<A_KC, B_KC, false>(gemm_lds + buf * GEMM_TILE_BYTES + a_base,
                                 gemm_lds + (2 + buf) * GEMM_TILE_BYTES + b_base, frag_half, frag_swz, acc, Ap, Bp, g, offa,
                                 offb, 0u, 0u, ra, rb);
    gemm_stage<A_KC>(gemm_lds + (buf ^ 1u) * GEMM_TILE_BYTES, ra, true, g.K, k_next);
    gemm_stage<B_KC>(gemm_lds + (2 + (buf ^ 1u)) * GEMM_TILE_BYTES, rb, true, g.K, k_next);
    __syncthreads();
  }
  if (n_steps > 0) {
    const u32 buf = (n_steps - 1) & 1u;
    gemm_step<A_KC, B_KC, false>(gemm_lds + buf * GEMM_TILE_BYTES + a_base,
                                 gemm_lds + (2 + buf) * GEMM_TILE_BYTES + b_base, frag_half, frag_swz, acc, Ap, Bp, g, offa,
                                 offb, 0u, 0u, ra, rb);
  }

  gemm_write_tile(g, g.n_split > 1 ? (int)EPI_PARTIAL : g.epilogue, acc, gemm_lds, m0 + wm * 128, n0 + wn * 128, split);
}

// Second launch of a split product: adds the partial tiles in the order of the splits and applies the epilogue.
__global__ void __launch_bounds__(BLOCK) k_gemm_reduce(GemmArgs g) {
  const u64 i4 = ((u64)blockIdx.x * BLOCK + threadIdx.x) * 4;  // 4 consecutive columns of one row
  const u64 mn = (u64)g.M * g.N;
  if (i4 >= mn) return;
  f4 s = ldg4(g.partial + i4);
  for (u32 sp = 1; sp < g.n_split; ++sp) {
    const f4 p = ldg4(g.partial + sp * mn + i4);
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  gemm_emit4(g, g.epilogue, (u32)(i4 / g.N), (u32)(i4 % g.N), s, 0);
}

// ---------------------------------------------------------------- host side

// How a product of this size is cut into work items: 256 x 256 tiles, and the number of ranges the
// contraction is split into.  The split is the one that minimises (rounds of 256 workgroups) x
// (contraction steps per work item + a fixed cost per item) + the cost of adding the partials.
struct GemmPlan {
  u32 tiles_m, tiles_n, n_split, k_per_split;
  size_t partial_bytes;  // fp32 scratch the split needs (0 when n_split == 1)
};

inline GemmPlan gemm_plan(u32 M, u32 N, u32 K, size_t partial_capacity) {
  GemmPlan p;
  p.tiles_m = (M + GEMM_BM - 1) / GEMM_BM;
  p.tiles_n = (N + GEMM_BN - 1) / GEMM_BN;
  const double tiles = (double)p.tiles_m * p.tiles_n, cus = 256.0;
  const u32 k_steps = (K + GEMM_BK - 1) / GEMM_BK;
  double best = 0.0;
  p.n_split = 1;
  for (u32 s = 1; s <= 32 && s <= k_steps; ++s) {
    const u32 steps_per = (k_steps + s - 1) / s;
    if (s > 1 && steps_per < 4) break;
    const size_t need = s > 1 ? (size_t)s * M * N * sizeof(float) : 0;
    if (need > partial_capacity) break;
    const double rounds = (double)(u64)((tiles * s + cus - 1) / cus);
    // unit: one contraction step of one tile (~3 us); fixed cost per item ~2 steps; the partials move
    // (s + 1) x M x N x 4 bytes at ~4 TB/s
    const double cost = rounds * (steps_per + 2.0) + (s > 1 ? (s + 1.0) * M * N * 4.0 / 4e12 / 3e-6 : 0.0);
    if (s == 1 || cost < best) {
      best = cost;
      p.n_split = s;
    }
  }
  const u32 steps_per = (k_steps + p.n_split - 1) / p.n_split;
  p.k_per_split = steps_per * GEMM_BK;
  p.n_split = (k_steps + steps_per - 1) / steps_per;  // no empty range at the end
  p.partial_bytes = p.n_split > 1 ? (size_t)p.n_split * M * N * sizeof(float) : 0;
  return p;
}

// Enqueues C = A B with the epilogue in `g` (operands, sizes, outputs and epilogue fields filled in by
// the caller).  partial: fp32 scratch of partial_capacity bytes for split products.
inline hipError_t gemm_enqueue(bool a_kc, bool b_kc, GemmArgs g, float* partial, size_t partial_capacity,
                               hipStream_t st) {
  if (g.M == 0 || g.N == 0 || g.K == 0) return hipErrorInvalidValue;
  if ((g.M | g.N | g.K | g.lda | g.ldb) % 8u != 0u) return hipErrorInvalidValue;
  // lanes address an operand with 32-bit byte offsets
  const u64 a_bytes = 2ull * g.lda * (a_kc ? g.M : g.K), b_bytes = 2ull * g.ldb * (b_kc ? g.N : g.K);
  if (a_bytes >= (1ull << 32) || b_bytes >= (1ull << 32)) return hipErrorInvalidValue;
  const GemmPlan p = gemm_plan(g.M, g.N, g.K, partial ? partial_capacity : 0);
  g.tiles_m = p.tiles_m;
  g.tiles_n = p.tiles_n;
  g.n_split = p.n_split;
  g.k_per_split = p.k_per_split;
  g.partial = partial;
  const u32 grid = p.tiles_m * p.tiles_n * p.n_split;
  hipError_t rc = hipSuccess;
#define CTR_GEMM_LAUNCH(AK, BK_, EA)                                                                              \
  do {                                                                                                            \
    static bool prepared = false; /* LDS beyond 64 KB has to be asked for once per kernel */                      \
    if (!prepared) {                                                                                              \
      rc = hipFuncSetAttribute((const void*)k_gemm_bf16<AK, BK_, EA>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                               (int)GEMM_LDS_BYTES);                                                              \
      if (rc != hipSuccess) return rc;                                                                            \
      prepared = true;                                                                                            \
    }                                                                                                             \
    hipLaunchKernelGGL((k_gemm_bf16<AK, BK_, EA>), dim3(grid), dim3(BLOCK), GEMM_LDS_BYTES, st, g.A, g.B, g);     \
  } while (0)
  const bool early = p.k_per_split / GEMM_BK >= 32;  // steps per work item
  const int which = (a_kc ? 4 : 0) | (b_kc ? 2 : 0) | (early ? 1 : 0);
  switch (which) {
    case 7: CTR_GEMM_LAUNCH(true, true, true); break;
    case 6: CTR_GEMM_LAUNCH(true, true, false); break;
    case 5: CTR_GEMM_LAUNCH(true, false, true); break;
    case 4: CTR_GEMM_LAUNCH(true, false, false); break;
    case 3: CTR_GEMM_LAUNCH(false, true, true); break;
    case 2: CTR_GEMM_LAUNCH(false, true, false); break;
    case 1: CTR_GEMM_LAUNCH(false, false, true); break;
    default: CTR_GEMM_LAUNCH(false, false, false); break;
  }
#undef CTR_GEMM_LAUNCH
  if (g.n_split > 1) {
    const u64 mn = (u64)g.M * g.N;
    hipLaunchKernelGGL(k_gemm_reduce, dim3((u32)((mn / 4 + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0, st, g);
  }
  return hipGetLastError();
}

}  // namespace ctr
