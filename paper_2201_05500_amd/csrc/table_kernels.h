// Key index (open addressing, insert-on-miss), row creation and the gather + per-segment sum.
//
// Paper: the per-GPU HBM hash table of Section 2.3 that holds the working
// parameters; Algorithm 1's insert_into_hash_table and pull steps; the state a
// new row starts from is Algorithm 2's "Initialize" line (m = 0, v = eps).
#pragma once
#include "common.h"

namespace ctr {

constexpr int RANK_ITEMS = 8;                     // occurrences per thread when ranking new keys
constexpr int RANK_TILE = BLOCK * RANK_ITEMS;     // 2048 occurrences per tile

// ---------------------------------------------------------------- table creation

__global__ void k_table_clear(DevHeader* hdr, Slot* slots, u64 n_slots, u32* row_state, u64 n_rows_cap) {
  const u64 tid = (u64)blockIdx.x * BLOCK + threadIdx.x;
  const u64 stride = (u64)gridDim.x * BLOCK;
  if (tid < 64) reinterpret_cast<u32*>(hdr)[tid] = 0;
  for (u64 i = tid; i < n_slots; i += stride) {
    Slot s;
    s.key = KEY_EMPTY;
    s.row = ROW_PENDING;
    s.first_p = 0xFFFFFFFFu;
    slots[i] = s;
  }
  for (u64 i = tid; i < n_rows_cap; i += stride) row_state[i] = 0;
}

// ---------------------------------------------------------------- probe / tentative insert

// One thread per key occurrence: linear probing from hash(key).  A hit on a
// committed slot yields the row id.  A miss claims the first free slot with a
// 64-bit compare-and-swap; the row id of such a slot is assigned later, so the
// occurrence records the slot index instead and lowers the slot's first_p to
// its own position (the smallest position wins: new rows are numbered in order
// of first occurrence).  The same launch checks the CSR offsets.
__global__ void k_probe_insert(DevHeader* hdr, Slot* slots, u32 slot_mask, const u64* __restrict__ keys,
                               u32 n_keys, const u32* __restrict__ offsets, u32 n_seg,
                               u32* __restrict__ occ_row) {
  if (hdr->status) return;
  const u32 tid = blockIdx.x * BLOCK + threadIdx.x;
  const u32 stride = gridDim.x * BLOCK;

  for (u32 g = tid; g <= n_seg; g += stride) {
    const u32 a = offsets[g];
    bool bad = (g == 0 && a != 0);
    if (g == n_seg)
      bad = bad || (a != n_keys);
    else
      bad = bad || (offsets[g + 1] < a);
    if (bad) atomicOr(&hdr->pull_err, ST_INVAL);
  }

  for (u32 p = tid; p < n_keys; p += stride) {
    const u64 key = keys[p];
    if (key == KEY_EMPTY) {
      atomicOr(&hdr->pull_err, ST_BADKEY);
      occ_row[p] = OCC_INVALID;
      continue;
    }
    u32 h = (u32)hash_key(key) & slot_mask;
    bool found = false;
    for (u32 probe = 0; probe <= slot_mask; ++probe) {
      u64 k = ld_relaxed(&slots[h].key);
      if (k == KEY_EMPTY) {
        const u64 old = atomicCAS(&slots[h].key, KEY_EMPTY, key);
        k = (old == KEY_EMPTY) ? key : old;
      }
      if (k == key) {
        found = true;
        break;
      }
      h = (h + 1) & slot_mask;
      if ((probe & 63u) == 63u && (ld_relaxed(&hdr->pull_err) & ST_FULL)) break;
    }
    if (!found) {  // every slot holds another key: more distinct keys than slots
      atomicOr(&hdr->pull_err, ST_FULL);
      occ_row[p] = OCC_INVALID;
      continue;
    }
    const u32 r = ld_relaxed(&slots[h].row);
    if (r == ROW_PENDING) {
      atomicMin(&slots[h].first_p, p);
      occ_row[p] = OCC_PEND_FLAG | h;
    } else {
      occ_row[p] = r;
    }
  }
}

// ---------------------------------------------------------------- ranking of new keys

__device__ __forceinline__ bool is_first_occurrence(const Slot* slots, u32 occ, u32 p) {
  if (occ == OCC_INVALID || !(occ & OCC_PEND_FLAG)) return false;
  return slots[occ & ~OCC_PEND_FLAG].first_p == p;
}

// Counts, per tile of RANK_TILE occurrences, those that are the first occurrence of a new key.
__global__ void k_count_first(const DevHeader* hdr, const Slot* __restrict__ slots,
                              const u32* __restrict__ occ_row, u32 n_keys, u32* __restrict__ tile_count) {
  if (hdr->status) return;
  __shared__ u32 lds[4];
  const u32 base = blockIdx.x * RANK_TILE + threadIdx.x * RANK_ITEMS;
  u32 cnt = 0;
#pragma unroll
  for (int i = 0; i < RANK_ITEMS; ++i) {
    const u32 p = base + i;
    if (p < n_keys) cnt += is_first_occurrence(slots, occ_row[p], p) ? 1u : 0u;
  }
  u32 total;
  block_exclusive_scan(cnt, lds, total);
  if (threadIdx.x == 0) tile_count[blockIdx.x] = total;
}

// One block: exclusive scan of the tile counts, capacity check, commit or roll back.
__global__ void k_scan_tiles(DevHeader* hdr, u32* __restrict__ tile_count, u32 n_tiles, u64 capacity_rows) {
  if (hdr->status) {  // an earlier call failed: this pull is a no-op
    if (threadIdx.x == 0) hdr->rollback = 0;
    return;
  }
  __shared__ u32 lds[4];
  u32 carry = 0;
  for (u32 t0 = 0; t0 < n_tiles; t0 += BLOCK) {
    const u32 t = t0 + threadIdx.x;
    const u32 v = (t < n_tiles) ? tile_count[t] : 0;
    u32 total;
    const u32 ex = block_exclusive_scan(v, lds, total);
    if (t < n_tiles) tile_count[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    u32 err = hdr->pull_err;
    const u32 base = hdr->n_rows;
    if ((u64)base + carry > capacity_rows) err |= ST_FULL;
    hdr->n_rows_base = base;
    hdr->pull_err = 0;
    hdr->n_unique = 0;
    if (err) {
      hdr->status = err;
      hdr->rollback = 1;
      hdr->n_new = 0;
    } else {
      hdr->rollback = 0;
      hdr->n_new = carry;
      hdr->n_rows = base + carry;
    }
  }
}

// Gives the first occurrence of every new key its row id (tile base + rank in
// occurrence order), or, when the pull failed, frees the slot again: clearing
// exactly the slots claimed by this pull restores the index as it was.
__global__ void k_assign_rows(const DevHeader* hdr, Slot* slots, const u32* __restrict__ occ_row, u32 n_keys,
                              const u32* __restrict__ tile_base, u64* __restrict__ row_key) {
  const u32 rollback = hdr->rollback;
  if (hdr->status && !rollback) return;
  __shared__ u32 lds[4];
  const u32 base = blockIdx.x * RANK_TILE + threadIdx.x * RANK_ITEMS;
  u32 slot_of[RANK_ITEMS];
  u32 cnt = 0;
#pragma unroll
  for (int i = 0; i < RANK_ITEMS; ++i) {
    const u32 p = base + i;
    slot_of[i] = 0xFFFFFFFFu;
    if (p < n_keys) {
      const u32 occ = occ_row[p];
      if (is_first_occurrence(slots, occ, p)) {
        slot_of[i] = occ & ~OCC_PEND_FLAG;
        ++cnt;
      }
    }
  }
  u32 total;
  u32 rank = block_exclusive_scan(cnt, lds, total);
  if (total == 0) return;
  const u32 row0 = hdr->n_rows_base + tile_base[blockIdx.x];
#pragma unroll
  for (int i = 0; i < RANK_ITEMS; ++i) {
    if (slot_of[i] == 0xFFFFFFFFu) continue;
    Slot* s = &slots[slot_of[i]];
    if (rollback) {
      s->first_p = 0xFFFFFFFFu;
      s->key = KEY_EMPTY;
    } else {
      const u32 row = row0 + rank++;
      s->row = row;
      row_key[row] = s->key;
    }
  }
}

// Writes the initial state of the rows created by this pull, in every replica:
// x = init(key, d), m = 0, v = eps, shared denominator = eps.
template <int LPR>
__global__ void k_init_rows(const DevHeader* hdr, const u64* __restrict__ row_key, float* values,
                            u64 replica_stride, u32 n_replicas, float* vhat, u32 D, u64 seed_mul,
                            float scale, float eps) {
  if (hdr->status) return;
  const u32 n_new = hdr->n_new, row_base = hdr->n_rows_base;
  const u32 c = threadIdx.x % LPR;
  const u32 groups = gridDim.x * (BLOCK / LPR);
  if (c * 4 >= D) return;
  for (u32 i = (blockIdx.x * BLOCK + threadIdx.x) / LPR; i < n_new; i += groups) {
    const u32 row = row_base + i;
    const u64 key = row_key[row];
    f4 x, z, e;
    x.x = init_value(seed_mul, key, 4 * c + 0, scale);
    x.y = init_value(seed_mul, key, 4 * c + 1, scale);
    x.z = init_value(seed_mul, key, 4 * c + 2, scale);
    x.w = init_value(seed_mul, key, 4 * c + 3, scale);
    z.x = z.y = z.z = z.w = 0.0f;
    e.x = e.y = e.z = e.w = eps;
    for (u32 j = 0; j < n_replicas; ++j) {
      float* b = values + j * replica_stride + (u64)row * 3 * D + 4 * c;
      stg4(b, x);
      stg4(b + D, z);
      stg4(b + 2 * D, e);
    }
    if (vhat) stg4(vhat + (u64)row * D + 4 * c, e);
  }
}

// Replaces "slot index, row pending" entries by the row id now that rows are assigned.
__global__ void k_resolve(const DevHeader* hdr, const Slot* __restrict__ slots, u32* __restrict__ occ_row,
                          u32 n_keys) {
  if (hdr->status) return;
  const u32 p = blockIdx.x * BLOCK + threadIdx.x;
  if (p >= n_keys) return;
  const u32 occ = occ_row[p];
  if (occ & OCC_PEND_FLAG) occ_row[p] = slots[occ & ~OCC_PEND_FLAG].row;
}

// ---------------------------------------------------------------- gather + per-segment sum

// One group of LPR lanes per segment, each lane owning 4 consecutive columns.
// pooled[g, :] = sum over the segment's occurrences of x[row, :], accumulated in
// binary64 in CSR order and rounded once.  Also records each occurrence's
// segment for the push.  Rows are [x | m | v] of 3*D floats.
template <int LPR>
__global__ void k_pool(const DevHeader* hdr, const u32* __restrict__ occ_row, u32* __restrict__ seg_of,
                       const u32* __restrict__ offsets, u32 n_seg, const float* __restrict__ values, u32 D,
                       float* __restrict__ pooled) {
  if (hdr->status) return;
  const u32 g = (blockIdx.x * BLOCK + threadIdx.x) / LPR;
  const u32 c = threadIdx.x % LPR;
  if (g >= n_seg) return;
  const bool col_ok = c * 4 < D;
  const u32 beg = offsets[g], end = offsets[g + 1];
  d4 acc = {0.0, 0.0, 0.0, 0.0};
  for (u32 p = beg; p < end; p += 4) {
    u32 r[4];
    f4 xv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (p + i < end) ? occ_row[p + i] : 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      xv[i].x = xv[i].y = xv[i].z = xv[i].w = 0.0f;
      if (p + i < end && col_ok) xv[i] = ldg4(values + (u64)r[i] * 3 * D + 4 * c);
    }
    if (c == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (p + i < end) seg_of[p + i] = g;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {  // adding +0.0 for the padded entries leaves the sum unchanged
      acc.x += (double)xv[i].x;
      acc.y += (double)xv[i].y;
      acc.z += (double)xv[i].z;
      acc.w += (double)xv[i].w;
    }
  }
  if (col_ok) {
    f4 o;
    o.x = (float)acc.x;
    o.y = (float)acc.y;
    o.z = (float)acc.z;
    o.w = (float)acc.w;
    stg4(pooled + (u64)g * D + 4 * c, o);
  }
}

}  // namespace ctr
