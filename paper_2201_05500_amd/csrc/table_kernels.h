// Key index (open addressing, insert-on-miss), row creation and the gather + per-segment sum.
//
// Paper: the per-GPU HBM hash table of Section 2.3 that holds the working
// parameters; Algorithm 1's insert_into_hash_table and pull steps; the state a
// new row starts from is Algorithm 2's "Initialize" line (m = 0, v = eps).
#pragma once
#include "common.h"

namespace ctr {


// ---------------------------------------------------------------- table creation

// keep_step_count: the number of accepted pushes (step count of the bias-corrected update) survives.
__global__ void k_table_clear(DevHeader* hdr, Slot* slots, u64 n_slots, u32* row_state, u64 n_rows_cap,
                              u32 keep_step_count) {
  const u64 tid = (u64)blockIdx.x * BLOCK + threadIdx.x;
  const u64 stride = (u64)gridDim.x * BLOCK;
  if (tid < 64 && !(keep_step_count && tid == HDR_WORD_N_PUSH)) reinterpret_cast<u32*>(hdr)[tid] = 0;
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

// One thread per key occurrence (a block takes a tile of 256 * items consecutive ones):
// linear probing from hash(key).  A hit on a committed slot yields the row id.  A miss claims
// the first free slot with a 64-bit compare-and-swap; the row id of such a slot is assigned
// later, so the occurrence records the slot index instead, lowers the slot's first_p to its
// own position (the smallest position wins: new rows are numbered in order of first
// occurrence) and is appended to its tile's list of pending occurrences (counted in LDS, so no
// global atomic is shared between blocks).  The same launch checks the CSR offsets and clears
// the bitmap of first occurrences.
constexpr int PROBE_MAX_ITEMS = 8;  // occurrences per thread: 8 for large batches, 1 for small ones (host's choice)

__global__ void __launch_bounds__(BLOCK)
k_probe_insert(DevHeader* hdr, Slot* slots, u32 slot_mask, const u64* __restrict__ keys, u32 n_keys,
               const u32* __restrict__ offsets, u32 n_seg, u32* __restrict__ occ_row,
               u32* __restrict__ first_bits, u32* __restrict__ pend_list, u32* __restrict__ tile_pending,
               u32 items) {
  if (hdr->status) return;
  __shared__ u32 n_pend;
  if (threadIdx.x == 0) n_pend = 0;
  __syncthreads();
  const u32 tile0 = blockIdx.x * (BLOCK * items);
  const int lane = lane_id();

#pragma unroll 1
  for (u32 it = 0; it < items; ++it) {
    const u32 p = tile0 + it * BLOCK + threadIdx.x;
    if (offsets != nullptr && p <= n_seg) {  // (a working-set load has no segments)
      const u32 a = offsets[p];
      bool bad = (p == 0 && a != 0);
      if (p == n_seg)
        bad = bad || (a != n_keys);
      else
        bad = bad || (offsets[p + 1] < a);
      if (bad) atomicOr(&hdr->pull_err, ST_INVAL);
    }

    bool pending = false;
    if (p < n_keys) {
      if ((p & 31u) == 0) first_bits[p >> 5] = 0;
      const u64 key = keys[p];
      u32 out = OCC_INVALID;
      if (key == KEY_EMPTY) {
        atomicOr(&hdr->pull_err, ST_BADKEY);
      } else {
        u32 h = (u32)hash_key(key) & slot_mask;
        bool found = false;
        u32 r = ROW_PENDING;
        for (u32 probe = 0; probe <= slot_mask; ++probe) {
          // One plain (cacheable) 16-byte load brings key and row id in a single request.  Slots
          // only ever go from free to taken inside this launch, so the worst a stale copy can
          // show is "free", and the compare-and-swap below then returns the key that is really
          // there; rows are assigned between launches, never inside this one, so a slot taken
          // during this launch has no row yet.
          const uint4 raw = *reinterpret_cast<const uint4*>(&slots[h]);
          u64 k = ((u64)raw.y << 32) | raw.x;
          r = raw.z;
          if (k == KEY_EMPTY) {
            const u64 old = atomicCAS(&slots[h].key, KEY_EMPTY, key);
            k = (old == KEY_EMPTY) ? key : old;
            r = ROW_PENDING;
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
        } else {
          if (r == ROW_PENDING) {
            // a popular new key has millions of occurrences: only those that can still lower
            // the minimum go to the atomic unit, the rest see a smaller value and pass
            if (ld_relaxed(&slots[h].first_p) > p) atomicMin(&slots[h].first_p, p);
            out = OCC_PEND_FLAG | h;
            pending = true;
          } else {
            out = r;
          }
        }
      }
      occ_row[p] = out;
    }

    // every lane of the wave is here again: one LDS atomic per wave reserves list entries
    const u64 bal = __ballot(pending);
    if (bal) {
      const int leader = __ffsll((long long)bal) - 1;
      u32 base = 0;
      if (lane == leader) base = atomicAdd(&n_pend, (u32)__popcll(bal));
      base = __shfl(base, leader, WAVE);
      if (pending) pend_list[tile0 + base + (u32)__popcll(bal & ((1ull << lane) - 1ull))] = p;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && tile0 < n_keys) tile_pending[blockIdx.x] = n_pend;  // blocks past the keys only check offsets
}

// ---------------------------------------------------------------- ranking of new keys

constexpr int BITS_TILE_WORDS = BLOCK;  // one bitmap word per thread: 8192 occurrences per tile

// Over the pending occurrences (one block per probe tile): marks those that are the first
// occurrence of their (new) key.  A probe tile owns whole words of the bitmap (its size is a
// multiple of 32 occurrences), so the bits are gathered in LDS and the words that hold any are
// stored plainly; the probe launch has zeroed the bitmap.
__global__ void k_flag_first(const DevHeader* hdr, const Slot* __restrict__ slots, const u32* __restrict__ occ_row,
                             const u32* __restrict__ pend_list, const u32* __restrict__ tile_pending,
                             u32 probe_tile, u32* __restrict__ first_bits) {
  if (hdr->status) return;
  const u32 cnt = tile_pending[blockIdx.x];
  if (cnt == 0) return;
  __shared__ u32 bits[PROBE_MAX_ITEMS * BLOCK / 32];
  const u32 tile_words = probe_tile / 32u, tile0 = blockIdx.x * probe_tile;
  for (u32 i = threadIdx.x; i < tile_words; i += BLOCK) bits[i] = 0;
  __syncthreads();
  for (u32 i = threadIdx.x; i < cnt; i += BLOCK) {
    const u32 p = pend_list[tile0 + i];
    const u32 h = occ_row[p] & ~OCC_PEND_FLAG;
    if (slots[h].first_p == p) atomicOr(&bits[(p - tile0) >> 5], 1u << (p & 31u));
  }
  __syncthreads();
  for (u32 i = threadIdx.x; i < tile_words; i += BLOCK)
    if (bits[i]) first_bits[(tile0 >> 5) + i] = bits[i];
}

// Number of first occurrences per tile of the bitmap.
__global__ void k_count_first(const DevHeader* hdr, const u32* __restrict__ first_bits, u32 n_words,
                              u32* __restrict__ tile_count) {
  if (hdr->status) return;
  __shared__ u32 lds[4];
  const u32 w = blockIdx.x * BITS_TILE_WORDS + threadIdx.x;
  const u32 cnt = (w < n_words) ? (u32)__popc(first_bits[w]) : 0u;
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
  const u32 per = (n_tiles + BLOCK - 1) / BLOCK;  // consecutive tiles per thread, one block-wide scan in all
  const u32 c0 = min(threadIdx.x * per, n_tiles), c1 = min(c0 + per, n_tiles);
  u32 sum = 0;
  for (u32 t = c0; t < c1; ++t) sum += tile_count[t];
  u32 carry;
  u32 ex = block_exclusive_scan(sum, lds, carry);
  for (u32 t = c0; t < c1; ++t) {
    const u32 v = tile_count[t];
    tile_count[t] = ex;
    ex += v;
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
// A block takes one tile of the bitmap: the words and their exclusive popcount prefix go to LDS,
// then every thread looks at 32 occurrences of its own (consecutive lanes, consecutive
// occurrences), so the slot accesses of a block are independent of each other.
__global__ void k_assign_rows(const DevHeader* hdr, Slot* slots, const u32* __restrict__ occ_row,
                              const u32* __restrict__ first_bits, u32 n_words, const u32* __restrict__ tile_base,
                              u64* __restrict__ row_key) {
  const u32 rollback = hdr->rollback;
  if (hdr->status && !rollback) return;
  __shared__ u32 lds[4];
  __shared__ u32 wbits[BITS_TILE_WORDS];
  __shared__ u32 wrank[BITS_TILE_WORDS];
  const u32 word0 = blockIdx.x * BITS_TILE_WORDS;
  const u32 mine = (word0 + threadIdx.x < n_words) ? first_bits[word0 + threadIdx.x] : 0u;
  u32 total;
  const u32 ex = block_exclusive_scan((u32)__popc(mine), lds, total);
  if (total == 0) return;
  wbits[threadIdx.x] = mine;
  wrank[threadIdx.x] = ex;
  __syncthreads();
  const u32 row0 = hdr->n_rows_base + tile_base[blockIdx.x];
  const u32 bit = threadIdx.x & 31u;
#pragma unroll 4
  for (u32 i = 0; i < 32; ++i) {
    const u32 word = i * (BLOCK / 32) + (threadIdx.x >> 5);
    const u32 b = wbits[word];
    if ((b >> bit) & 1u) {
      const u32 p = (word0 + word) * 32u + bit;
      Slot* s = &slots[occ_row[p] & ~OCC_PEND_FLAG];
      if (rollback) {
        s->first_p = 0xFFFFFFFFu;
        s->key = KEY_EMPTY;
      } else {
        const u32 row = row0 + wrank[word] + (u32)__popc(b & ((1u << bit) - 1u));
        s->row = row;
        row_key[row] = s->key;
      }
    }
  }
}

// Writes the initial state of the rows created by this pull, in every replica:
// x = init(key, d); first moment 0 (rows that have one); second moment / AdaGrad accumulator
// = v0 (eps per Algorithm 2's "Initialize", 0 for the bias-corrected form); shared denominator = v0.
// rf = floats per row (3*D with a first moment, 2*D without).
template <int LPR>
__global__ void k_init_rows(const DevHeader* hdr, const u64* __restrict__ row_key, float* values,
                            u64 replica_stride, u32 n_replicas, float* vhat, u32 D, u32 rf, u64 seed_mul,
                            float scale, float v0) {
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
    e.x = e.y = e.z = e.w = v0;
    for (u32 j = 0; j < n_replicas; ++j) {
      float* b = values + j * replica_stride + (u64)row * rf + 4 * c;
      stg4(b, x);
      if (rf == 3 * D) {
        stg4(b + D, z);
        stg4(b + 2 * D, e);
      } else {
        stg4(b + D, e);
      }
    }
    if (vhat) stg4(vhat + (u64)row * D + 4 * c, e);
  }
}

// Replaces "slot index, row pending" entries by the row id now that rows are assigned
// (one block per probe tile, over its list of pending occurrences).
__global__ void k_resolve(const DevHeader* hdr, const Slot* __restrict__ slots, u32* __restrict__ occ_row,
                          const u32* __restrict__ pend_list, const u32* __restrict__ tile_pending,
                          u32 probe_tile) {
  if (hdr->status) return;
  const u32 cnt = tile_pending[blockIdx.x];
  for (u32 i = threadIdx.x; i < cnt; i += BLOCK) {
    const u32 p = pend_list[blockIdx.x * probe_tile + i];
    occ_row[p] = slots[occ_row[p] & ~OCC_PEND_FLAG].row;
  }
}

// ---------------------------------------------------------------- working-set load / collection

// After the keys of a working set have been looked up or inserted (occ_row[p] = row of keys[p]):
// overwrites the state of those rows, in every replica, with the values supplied by the caller
// (the shared denominator, where there is one, is set to v).  m_src may be null for rows without
// a first moment.
template <int LPR>
__global__ void k_load_rows(const DevHeader* hdr, const u32* __restrict__ occ_row, u32 n, float* values,
                            u64 replica_stride, u32 n_replicas, float* vhat, u32 D, u32 rf,
                            const float* __restrict__ x_src, const float* __restrict__ m_src,
                            const float* __restrict__ v_src) {
  if (hdr->status) return;
  const u64 p64 = ((u64)blockIdx.x * BLOCK + threadIdx.x) / LPR;  // n * LPR threads can pass 2^32
  const u32 c = threadIdx.x % LPR;
  if (p64 >= n || c * 4 >= D) return;
  const u32 p = (u32)p64;
  const u32 row = occ_row[p];
  const f4 x = ldg4(x_src + (u64)p * D + 4 * c);
  const f4 v = ldg4(v_src + (u64)p * D + 4 * c);
  f4 m = {0.0f, 0.0f, 0.0f, 0.0f};
  if (rf == 3 * D) m = ldg4(m_src + (u64)p * D + 4 * c);
  for (u32 j = 0; j < n_replicas; ++j) {
    float* b = values + j * replica_stride + (u64)row * rf + 4 * c;
    stg4(b, x);
    if (rf == 3 * D) {
      stg4(b + D, m);
      stg4(b + 2 * D, v);
    } else {
      stg4(b + D, v);
    }
  }
  if (vhat) stg4(vhat + (u64)row * D + 4 * c, v);
}

// Lookup without insert for every occurrence of a batch (prediction): occ_row[p] = row of keys[p],
// or OCC_INVALID if the key is not in the table.  Checks keys and offsets like the training probe;
// what it finds goes to pull_err and is folded into the status by k_lookup_commit.
__global__ void __launch_bounds__(BLOCK)
k_lookup(DevHeader* hdr, const Slot* __restrict__ slots, u32 slot_mask, const u64* __restrict__ keys, u32 n_keys,
         const u32* __restrict__ offsets, u32 n_seg, u32* __restrict__ occ_row) {
  if (hdr->status) return;
  const u32 p = blockIdx.x * BLOCK + threadIdx.x;
  if (p <= n_seg) {
    const u32 a = offsets[p];
    bool bad = (p == 0 && a != 0);
    if (p == n_seg)
      bad = bad || (a != n_keys);
    else
      bad = bad || (offsets[p + 1] < a);
    if (bad) atomicOr(&hdr->pull_err, ST_INVAL);
  }
  if (p >= n_keys) return;
  const u64 key = keys[p];
  u32 out = OCC_INVALID;
  if (key == KEY_EMPTY) {
    atomicOr(&hdr->pull_err, ST_BADKEY);
  } else {
    u32 h = (u32)hash_key(key) & slot_mask;
    for (u32 probe = 0; probe <= slot_mask; ++probe) {
      const uint4 raw = *reinterpret_cast<const uint4*>(&slots[h]);  // key and row id in one request
      const u64 k = ((u64)raw.y << 32) | raw.x;
      if (k == key) {
        out = raw.z;
        break;
      }
      if (k == KEY_EMPTY) break;
      h = (h + 1) & slot_mask;
    }
  }
  occ_row[p] = out;
}

__global__ void k_lookup_commit(DevHeader* hdr) {
  if (threadIdx.x == 0 && blockIdx.x == 0 && !hdr->status) {
    hdr->status = hdr->pull_err;
    hdr->pull_err = 0;
  }
}

// Pure lookup (no insert) of n keys and copy of their rows of one replica to dense arrays; a key
// that is not in the table gets found = 0 and zeros.
template <int LPR>
__global__ void k_collect_rows(const DevHeader* hdr, const Slot* __restrict__ slots, u32 slot_mask,
                               const u64* __restrict__ keys, u32 n, const float* __restrict__ values, u32 D,
                               u32 rf, float* __restrict__ x_dst, float* __restrict__ m_dst,
                               float* __restrict__ v_dst, u32* __restrict__ found) {
  if (hdr->status) return;
  const u64 p64 = ((u64)blockIdx.x * BLOCK + threadIdx.x) / LPR;  // n * LPR threads can pass 2^32
  const u32 c = threadIdx.x % LPR;
  if (p64 >= n) return;
  const u32 p = (u32)p64;
  const u64 key = keys[p];
  u32 row = ROW_PENDING;
  if (key != KEY_EMPTY) {
    u32 h = (u32)hash_key(key) & slot_mask;
    for (u32 probe = 0; probe <= slot_mask; ++probe) {  // every lane of the group walks the same slots
      const u64 k = slots[h].key;
      if (k == key) {
        row = slots[h].row;
        break;
      }
      if (k == KEY_EMPTY) break;
      h = (h + 1) & slot_mask;
    }
  }
  const bool hit = row != ROW_PENDING;
  if (c == 0 && found) found[p] = hit ? 1u : 0u;
  if (c * 4 >= D) return;
  f4 x = {0.0f, 0.0f, 0.0f, 0.0f}, m = x, v = x;
  if (hit) {
    const float* b = values + (u64)row * rf + 4 * c;
    x = ldg4(b);
    if (rf == 3 * D) {
      m = ldg4(b + D);
      v = ldg4(b + 2 * D);
    } else {
      v = ldg4(b + D);
    }
  }
  if (x_dst) stg4(x_dst + (u64)p * D + 4 * c, x);
  if (m_dst) stg4(m_dst + (u64)p * D + 4 * c, m);
  if (v_dst) stg4(v_dst + (u64)p * D + 4 * c, v);
}

// ---------------------------------------------------------------- gather + per-segment sum

// A block takes POOL_TILE consecutive segments and stages their CSR boundaries in LDS.
// First all threads record, for every occurrence of the tile, the segment it belongs to
// (binary search in the staged boundaries; coalesced writes) - the push needs it.
// Then each group of LPR lanes (a lane owns 4 consecutive columns) sums its segments, two
// at a time so that up to 8 independent row loads are in flight per group:
// pooled[g, :] = sum over the segment's occurrences of x[row, :], in CSR order, binary32
// inside a batch of 4 consecutive occurrences and binary64 across batches, rounded once
// (error <= 3 * 2^-24 * sum |x|).  A row is rf floats and starts with x.
#ifndef CTR_POOL_NT_OUT
#define CTR_POOL_NT_OUT 1  // the pooled output (written once, read by the next stage) leaves with the non-temporal hint
#endif
constexpr int POOL_NS = 2;      // segments a group works on at once
constexpr int POOL_ROUNDS = 2;  // such pairs per group

// OUT: 1 = fp32 output, 2 = bf16 output, 3 = both; + 4 = lookup-only input, where an occurrence may have
// no row (compile-time, so the common fp32-only training kernel carries none of the other cases).
template <int LPR, int OUT>
__device__ __forceinline__ void pool_body(const DevHeader* hdr, const u32* __restrict__ occ_row,
                                          u32* __restrict__ seg_of, const u32* __restrict__ offsets, u32 n_seg,
                                          const float* __restrict__ values, u32 D, u32 rf,
                                          float* __restrict__ pooled, bf16_t* __restrict__ pooled_bf16) {
  if (hdr->status) return;
  constexpr int GROUPS = BLOCK / LPR;
  constexpr int TILE = GROUPS * POOL_NS * POOL_ROUNDS;
  __shared__ u32 off_lds[TILE + 1];
  const u32 tile_g0 = blockIdx.x * TILE;
  const u32 tile_n = min((u32)TILE, n_seg - tile_g0);
  for (u32 i = threadIdx.x; i <= tile_n; i += BLOCK) off_lds[i] = offsets[tile_g0 + i];
  __syncthreads();

  const u32 P0 = off_lds[0], P1 = off_lds[tile_n];
  for (u32 p = P0 + threadIdx.x; p < P1; p += BLOCK) {
    u32 lo = 0, hi = tile_n;  // last l with off[l] <= p (skips empty segments)
    while (hi - lo > 1) {
      const u32 mid = (lo + hi) >> 1;
      if (off_lds[mid] <= p) lo = mid; else hi = mid;
    }
    seg_of[p] = tile_g0 + lo;
  }

  const u32 grp = threadIdx.x / LPR, c = threadIdx.x % LPR;
  const bool col_ok = c * 4 < D;
#pragma unroll
  for (int rnd = 0; rnd < POOL_ROUNDS; ++rnd) {
    u32 beg[POOL_NS], end[POOL_NS];
    d4 acc[POOL_NS];
    u32 maxlen = 0;
#pragma unroll
    for (int s = 0; s < POOL_NS; ++s) {
      const u32 l = (rnd * POOL_NS + s) * GROUPS + grp;
      beg[s] = l < tile_n ? off_lds[l] : 0u;
      end[s] = l < tile_n ? off_lds[l + 1] : 0u;
      acc[s] = d4{0.0, 0.0, 0.0, 0.0};
      maxlen = max(maxlen, end[s] - beg[s]);
    }
    u32 win[POOL_NS];  // lane c of the group holds the row id of occurrence (window start + c)
    for (u32 k = 0; k < maxlen; k += 4) {
      u32 r[POOL_NS][4];
      f4 xv[POOL_NS][4];
      if constexpr (LPR >= 4) {
        // one coalesced load per group brings the row ids of the next LPR occurrences (a whole
        // segment, usually); they are handed out by shuffles: a quarter of the memory requests
        // of one broadcast load per occurrence
        if (k % LPR == 0) {
#pragma unroll
          for (int s = 0; s < POOL_NS; ++s) win[s] = (beg[s] + k + c < end[s]) ? occ_row[beg[s] + k + c] : 0u;
        }
#pragma unroll
        for (int s = 0; s < POOL_NS; ++s)
#pragma unroll
          for (int i = 0; i < 4; ++i) r[s][i] = __shfl(win[s], (int)((k + i) % LPR), LPR);
      } else {
#pragma unroll
        for (int s = 0; s < POOL_NS; ++s)
#pragma unroll
          for (int i = 0; i < 4; ++i) r[s][i] = (beg[s] + k + i < end[s]) ? occ_row[beg[s] + k + i] : 0u;
      }
#pragma unroll
      for (int s = 0; s < POOL_NS; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          xv[s][i].x = xv[s][i].y = xv[s][i].z = xv[s][i].w = 0.0f;
          bool take = beg[s] + k + i < end[s] && col_ok;
          if constexpr (OUT & 4) take = take && r[s][i] != OCC_INVALID;  // lookup-only: absent keys add nothing
          if (take) xv[s][i] = ldg4(values + (u64)r[s][i] * rf + 4 * c);
        }
#pragma unroll
      for (int s = 0; s < POOL_NS; ++s) {  // padded entries add +0.0
        f4 f = xv[s][0];
#pragma unroll
        for (int i = 1; i < 4; ++i) {
          f.x += xv[s][i].x; f.y += xv[s][i].y; f.z += xv[s][i].z; f.w += xv[s][i].w;
        }
        acc[s].x += (double)f.x; acc[s].y += (double)f.y; acc[s].z += (double)f.z; acc[s].w += (double)f.w;
      }
    }
#pragma unroll
    for (int s = 0; s < POOL_NS; ++s) {
      const u32 l = (rnd * POOL_NS + s) * GROUPS + grp;
      if (l < tile_n && col_ok) {
        f4 o = {(float)acc[s].x, (float)acc[s].y, (float)acc[s].z, (float)acc[s].w};
#if CTR_POOL_NT_OUT
        if constexpr (OUT & 1) stg4_stream(pooled + (u64)(tile_g0 + l) * D + 4 * c, o);
#else
        if constexpr (OUT & 1) stg4(pooled + (u64)(tile_g0 + l) * D + 4 * c, o);
#endif
        if constexpr (OUT & 2) stg4_bf16(pooled_bf16 + (u64)(tile_g0 + l) * D + 4 * c, o);  // the fp32 value, rounded again
      }
    }
  }
}

#define CTR_POOL_ARGS                                                                                       \
  const DevHeader *hdr, const u32 *__restrict__ occ_row, u32 *__restrict__ seg_of,                          \
      const u32 *__restrict__ offsets, u32 n_seg, const float *__restrict__ values, u32 D, u32 rf,          \
      float *__restrict__ pooled, bf16_t *__restrict__ pooled_bf16
#define CTR_DEFINE_POOL(NAME, OUT)                                                            \
  template <int LPR>                                                                          \
  __global__ void __launch_bounds__(BLOCK) NAME(CTR_POOL_ARGS) {                              \
    pool_body<LPR, OUT>(hdr, occ_row, seg_of, offsets, n_seg, values, D, rf, pooled, pooled_bf16); \
  }
CTR_DEFINE_POOL(k_pool, 1)
CTR_DEFINE_POOL(k_pool_bf16, 2)
CTR_DEFINE_POOL(k_pool_both, 3)
CTR_DEFINE_POOL(k_pool_lookup, 5)
CTR_DEFINE_POOL(k_pool_lookup_bf16, 6)
CTR_DEFINE_POOL(k_pool_lookup_both, 7)

}  // namespace ctr
