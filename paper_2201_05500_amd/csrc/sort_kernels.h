// Grouping of key occurrences by row id: a stable least-significant-digit radix sort of
// (row id, segment id) pairs, hand-written for wave64 and a 160 KB LDS.
//
// Paper: the push of Algorithm 1 updates each referenced parameter once per
// mini-batch, so the occurrences of one key must be brought together before
// their gradients can be summed (the "union of the referenced parameters" of
// Section 2.3, here formed on the GPU).  Row ids are dense small integers
// (ceil(log2 R) bits), so sorting them costs half the passes of sorting the
// 64-bit keys.
//
// One pass = three launches:
//   k_sort_hist    per-chunk digit histogram           -> hist[digit][chunk]
//   k_sort_scan    per digit: exclusive scan over chunks, digit totals
//   k_sort_scatter per chunk: for each 4096-element sub-tile, rank elements
//                  per digit inside each wave with ballots (stable), counting-
//                  sort the sub-tile in LDS, then write each digit's run to
//                  its place; runs are contiguous, so the writes coalesce.
#pragma once
#include "common.h"

namespace ctr {

#ifndef CTR_SORT_ITEMS
#define CTR_SORT_ITEMS 16
#endif
constexpr int SORT_ITEMS = CTR_SORT_ITEMS;
constexpr int SORT_TILE = BLOCK * SORT_ITEMS;  // 4096
#ifndef CTR_SORT_MAX_CHUNKS
#define CTR_SORT_MAX_CHUNKS 4096
#endif
constexpr int SORT_MAX_CHUNKS = CTR_SORT_MAX_CHUNKS;
constexpr int RADIX = 256;
#ifndef CTR_HIST_COPIES
#define CTR_HIST_COPIES 4
#endif
constexpr int HIST_COPIES = CTR_HIST_COPIES;  // power of two

struct SortGeom {
  u32 n;            // elements
  u32 n_chunks;     // blocks of the histogram / scatter launches
  u32 chunk_elems;  // multiple of SORT_TILE
};

__global__ void k_sort_hist(const DevHeader* hdr, const u32* __restrict__ keys, SortGeom geo, u32 shift,
                            u32 digit_mask, u32* __restrict__ hist) {
  if (hdr->status) return;
  // HIST_COPIES histograms per wave, chosen by lane: a popular digit (row ids of popular keys share
  // their high bits) would otherwise serialise all 64 lanes on one LDS address
  __shared__ u32 h[4 * HIST_COPIES][RADIX];
#pragma unroll
  for (int i = 0; i < 4 * HIST_COPIES; ++i) h[i][threadIdx.x] = 0;
  __syncthreads();
  const u32 beg = blockIdx.x * geo.chunk_elems;  // multiple of SORT_TILE, so 16-byte aligned
  const u32 end = min(beg + geo.chunk_elems, geo.n);
  u32* mine = h[wave_id() * HIST_COPIES + (lane_id() & (HIST_COPIES - 1))];
  for (u32 e = beg + threadIdx.x * 4; e < end; e += BLOCK * 4) {
    if (e + 4 <= end) {
      const uint4 k4 = *reinterpret_cast<const uint4*>(keys + e);
      const u32 d0 = (k4.x >> shift) & digit_mask, d1 = (k4.y >> shift) & digit_mask;
      const u32 d2 = (k4.z >> shift) & digit_mask, d3 = (k4.w >> shift) & digit_mask;
      // the digit of the wave's first key is counted with ballots (one add for the whole wave):
      // under a popular digit that takes most of the keys away from the LDS atomics
      const u32 ref = (u32)__builtin_amdgcn_readfirstlane((int)d0);
      const u32 n_ref = (u32)(__popcll(__ballot(d0 == ref)) + __popcll(__ballot(d1 == ref)) +
                              __popcll(__ballot(d2 == ref)) + __popcll(__ballot(d3 == ref)));
      if (d0 != ref) atomicAdd(&mine[d0], 1u);
      if (d1 != ref) atomicAdd(&mine[d1], 1u);
      if (d2 != ref) atomicAdd(&mine[d2], 1u);
      if (d3 != ref) atomicAdd(&mine[d3], 1u);
      if (lane_id() == __ffsll((long long)__ballot(true)) - 1) atomicAdd(&mine[ref], n_ref);  // first lane that is here
    } else {
      for (u32 j = e; j < end; ++j) atomicAdd(&mine[(keys[j] >> shift) & digit_mask], 1u);
    }
  }
  __syncthreads();
  u32 total = 0;
#pragma unroll
  for (int i = 0; i < 4 * HIST_COPIES; ++i) total += h[i][threadIdx.x];
  hist[threadIdx.x * geo.n_chunks + blockIdx.x] = total;
}

// grid = RADIX blocks; block d turns hist[d][0..n_chunks) into exclusive prefix sums.
__global__ void k_sort_scan(const DevHeader* hdr, u32* __restrict__ hist, u32 n_chunks,
                            u32* __restrict__ digit_total) {
  if (hdr->status) return;
  __shared__ u32 lds[4];
  u32* row = hist + blockIdx.x * n_chunks;
  const u32 per = (n_chunks + BLOCK - 1) / BLOCK;  // consecutive entries per thread
  const u32 c0 = threadIdx.x * per;
  const u32 c1 = min(c0 + per, n_chunks);
  u32 s = 0;
  for (u32 i = c0; i < c1; ++i) s += row[i];
  u32 total;
  u32 ex = block_exclusive_scan(s, lds, total);
  for (u32 i = c0; i < c1; ++i) {
    const u32 v = row[i];
    row[i] = ex;
    ex += v;
  }
  if (threadIdx.x == 0) digit_total[blockIdx.x] = total;
}

__global__ void __launch_bounds__(BLOCK)
k_sort_scatter(const DevHeader* hdr, const u32* __restrict__ keys_in, const u32* __restrict__ vals_in,
               u32* __restrict__ keys_out, u32* __restrict__ vals_out, SortGeom geo, u32 shift,
               u32 digit_mask, const u32* __restrict__ hist, const u32* __restrict__ digit_total) {
  if (hdr->status) return;
  __shared__ u32 scan_lds[4];
  __shared__ u32 gbase[RADIX];        // next global position of each digit for this chunk
  __shared__ u32 whist[4][RADIX];     // per-wave digit counts, then per-wave local bases
  __shared__ u32 dstart[RADIX];       // sub-tile-local start of each digit
  __shared__ u32 dcount[RADIX];
  __shared__ u32 lkeys[SORT_TILE];
  __shared__ u32 lvals[SORT_TILE];

  const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
  {
    u32 total;
    const u32 ex = block_exclusive_scan(digit_total[tid], scan_lds, total);
    gbase[tid] = ex + hist[tid * geo.n_chunks + blockIdx.x];
  }
  const u32 chunk_beg = blockIdx.x * geo.chunk_elems;
  const u32 chunk_end = min(chunk_beg + geo.chunk_elems, geo.n);
  const u64 lanes_below = (1ull << lane) - 1ull;

  for (u32 sub = chunk_beg; sub < chunk_end; sub += SORT_TILE) {
    const u32 n_valid = min((u32)SORT_TILE, chunk_end - sub);
#pragma unroll
    for (int i = 0; i < 4; ++i) whist[i][tid] = 0;
    __syncthreads();

    u32 k[SORT_ITEMS], v[SORT_ITEMS], rank[SORT_ITEMS];
    volatile u32* my_hist = whist[w];
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
      const u32 local = w * (SORT_TILE / 4) + i * WAVE + lane;  // waves own consecutive quarters
      const bool valid = local < n_valid;
      k[i] = valid ? keys_in[sub + local] : 0u;
      v[i] = valid ? vals_in[sub + local] : 0u;
    }
#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
      const u32 local = w * (SORT_TILE / 4) + i * WAVE + lane;
      const bool valid = local < n_valid;
      const u32 d = (k[i] >> shift) & digit_mask;  // 0 for lanes past the end (k = 0)
      // lanes whose digit equals mine: for every bit, the ballot of that bit XNOR my bit (m is
      // 0 or ~0); the disagreements are OR-ed per 32-bit half, lanes past the end masked at the end
      u32 diff_lo = 0, diff_hi = 0;
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        const u32 m = (u32)__builtin_amdgcn_sbfe((int)d, b, 1);
        const u64 bal = __builtin_amdgcn_ballot_w64(m != 0u);
        diff_lo |= (u32)bal ^ m;
        diff_hi |= (u32)(bal >> 32) ^ m;
      }
      const u64 same = __ballot(valid) & ~(((u64)diff_hi << 32) | diff_lo);
      // lanes of `same` hold digit d; the lowest of them bumps the wave's counter
      const int leader = __ffsll((long long)same) - 1;
      u32 before = 0;
      if (valid && lane == leader) {
        before = my_hist[d];
        my_hist[d] = before + (u32)__popcll(same);
      }
      before = __shfl(before, leader < 0 ? 0 : leader, WAVE);
      rank[i] = before + (u32)__popcll(same & lanes_below);
    }
    __syncthreads();

    {  // digit-major, wave-minor exclusive scan of the counts
      const u32 c0 = whist[0][tid], c1 = whist[1][tid], c2 = whist[2][tid], c3 = whist[3][tid];
      u32 total;
      const u32 ex = block_exclusive_scan(c0 + c1 + c2 + c3, scan_lds, total);
      dstart[tid] = ex;
      dcount[tid] = c0 + c1 + c2 + c3;
      whist[0][tid] = ex;
      whist[1][tid] = ex + c0;
      whist[2][tid] = ex + c0 + c1;
      whist[3][tid] = ex + c0 + c1 + c2;
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < SORT_ITEMS; ++i) {
      const u32 local = w * (SORT_TILE / 4) + i * WAVE + lane;
      if (local < n_valid) {
        const u32 d = (k[i] >> shift) & digit_mask;
        const u32 pos = whist[w][d] + rank[i];
        lkeys[pos] = k[i];
        lvals[pos] = v[i];
      }
    }
    __syncthreads();

    for (u32 j = tid; j < n_valid; j += BLOCK) {
      const u32 kk = lkeys[j];
      const u32 d = (kk >> shift) & digit_mask;
      const u32 pos = gbase[d] + (j - dstart[d]);
      keys_out[pos] = kk;
      vals_out[pos] = lvals[j];
    }
    __syncthreads();
    gbase[tid] += dcount[tid];
    // the barrier at the top of the next iteration orders this against its readers
  }
}

}  // namespace ctr
