// Host side of the C ABI declared in include/ctr_sparse.h: argument checks, memory layout,
// kernel launches.  No arithmetic of the method happens on the host (hyper-parameters are
// promoted to binary64 and complemented here, nothing else).
#include "../../include/ctr_sparse.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include "push_kernels.h"
#include "sort_kernels.h"
#include "table_kernels.h"

using namespace ctr;

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline u64 pow2ceil(u64 x) {
  u64 p = 1;
  while (p < x) p <<= 1;
  return p;
}

struct TableLayout {
  u64 n_slots;
  size_t off_hdr, off_slots, off_row_key, off_row_state, off_values, off_vhat, total;
  u64 replica_stride;  // floats between replicas
};

bool config_ok(const ctr_config* c) {
  if (!c) return false;
  if (c->dim == 0 || c->dim % 4 != 0 || c->dim > 256) return false;
  if (c->capacity_rows == 0 || c->capacity_rows > (1ull << 30)) return false;
  if (c->n_replicas == 0 || c->n_replicas > 31) return false;
  if (!(c->load_factor >= 0.0f) || c->load_factor > 0.9f) return false;
  const uint32_t known = CTR_F_KSTEP | CTR_F_ADAGRAD | CTR_F_KSTEP_PROSE | CTR_F_BIAS_CORRECTION;
  if (c->flags & ~known) return false;
  if ((c->flags & CTR_F_KSTEP_PROSE) && !(c->flags & CTR_F_KSTEP)) return false;
  if ((c->flags & CTR_F_ADAGRAD) && (c->flags & ~CTR_F_ADAGRAD)) return false;          // no replicas, no variants
  if ((c->flags & CTR_F_BIAS_CORRECTION) && (c->flags & ~CTR_F_BIAS_CORRECTION)) return false;
  if (!(c->flags & CTR_F_KSTEP) && c->n_replicas != 1) return false;                    // replicas exist to be merged
  if (!(c->lr > 0.0f) || !(c->beta1 >= 0.0f && c->beta1 < 1.0f) || !(c->beta2 >= 0.0f && c->beta2 < 1.0f) ||
      !(c->eps > 0.0f) || !(c->init_std >= 0.0f))
    return false;
  return true;
}

bool table_layout(const ctr_config* c, TableLayout* L) {
  if (!config_ok(c)) return false;
  const double lf = c->load_factor == 0.0f ? 0.5 : (double)c->load_factor;
  u64 want = (u64)std::ceil((double)c->capacity_rows / lf);
  L->n_slots = std::max<u64>(pow2ceil(want), 64);
  if (L->n_slots > (1ull << 30)) return false;
  const u64 R = c->capacity_rows, D = c->dim, W = c->n_replicas;
  size_t o = 0;
  L->off_hdr = o; o += align256(sizeof(DevHeader));
  L->off_slots = o; o += align256(L->n_slots * sizeof(Slot));
  L->off_row_key = o; o += align256(R * sizeof(u64));
  L->off_row_state = o; o += align256(R * sizeof(u32));
  L->off_values = o;
  const u64 n_state = (c->flags & CTR_F_ADAGRAD) ? 2 : 3;  // [x | G] or [x | m | v]
  L->replica_stride = (align256(R * n_state * D * sizeof(float))) / sizeof(float);
  o += L->replica_stride * sizeof(float) * W;
  L->off_vhat = o;
  if ((c->flags & CTR_F_KSTEP) && !(c->flags & CTR_F_KSTEP_PROSE)) o += align256(R * D * sizeof(float));
  L->total = o;
  return true;
}

struct WorkLayout {
  u32 n_bit_words, n_bit_tiles, probe_items, probe_tile, n_probe_tiles, span, n_spans, n_span_blocks;
  SortGeom geo;
  size_t off_occ_row, off_seg_of, off_ka, off_va, off_kb, off_vb, off_hist, off_digit_total, off_tile_count, off_first_bits, off_pend_list, off_tile_pending,
      off_head, off_tail, off_block_head, off_span_flags, off_span_rows, total;
};

// How a list of n elements is cut into the chunks the sort's launches work on.
SortGeom sort_geom(u64 n) {
  const u64 tiles = (n + SORT_TILE - 1) / SORT_TILE;
  const u64 chunks = std::min<u64>(std::max<u64>(tiles, 1), SORT_MAX_CHUNKS);
  const u64 per = (n + chunks - 1) / chunks;
  const u64 chunk_elems = std::max<u64>(((per + SORT_TILE - 1) / SORT_TILE) * SORT_TILE, SORT_TILE);
  SortGeom g;
  g.n = (u32)n;
  g.chunk_elems = (u32)chunk_elems;
  g.n_chunks = (u32)std::max<u64>((n + chunk_elems - 1) / chunk_elems, 1);
  return g;
}

// force_span / force_items: 0 = chosen by batch size; otherwise the geometry a test asks for.
void work_layout(u32 D, u64 n_keys, WorkLayout* L, u32 force_span = 0, u32 force_items = 0) {
  const u64 n = n_keys;
  L->n_bit_words = (u32)((n + 31) / 32);
  L->n_bit_tiles = (L->n_bit_words + BITS_TILE_WORDS - 1) / BITS_TILE_WORDS;
  // shorter spans for smaller batches: the span walk is sequential, so parallelism = n / span groups
  L->span = n >= (8u << 20) ? 128u : n >= (4u << 20) ? 64u : n >= (2u << 20) ? 32u : 16u;
  if (force_span) L->span = force_span;
  L->n_spans = (u32)((n + L->span - 1) / L->span);
  L->n_span_blocks = (L->n_spans + SPANS_PER_BLOCK - 1) / SPANS_PER_BLOCK;
  L->geo = sort_geom(n);
  size_t o = 0;
  const size_t arr = align256(n * sizeof(u32));
  L->off_occ_row = o; o += arr;
  L->off_seg_of = o; o += arr;
  L->off_ka = o; o += arr;
  L->off_va = o; o += arr;
  L->off_kb = o; o += arr;
  L->off_vb = o; o += arr;
  L->off_hist = o; o += align256((size_t)RADIX * SORT_MAX_CHUNKS * sizeof(u32));
  L->off_digit_total = o; o += align256(RADIX * sizeof(u32));
  L->off_tile_count = o; o += align256(((size_t)L->n_bit_tiles + 1) * sizeof(u32));
  L->off_first_bits = o; o += align256(((size_t)L->n_bit_words + 1) * sizeof(u32));
  L->probe_items = n >= (4u << 20) ? PROBE_MAX_ITEMS : 1;
  if (force_items) L->probe_items = force_items;
  L->probe_tile = BLOCK * L->probe_items;
  L->n_probe_tiles = (u32)((n + L->probe_tile - 1) / L->probe_tile);
  L->off_pend_list = o; o += align256(((size_t)L->n_probe_tiles + 1) * L->probe_tile * sizeof(u32));
  L->off_tile_pending = o; o += align256(((size_t)L->n_probe_tiles + 1) * sizeof(u32));
  L->off_head = o; o += align256((size_t)L->n_spans * D * sizeof(double));
  L->off_tail = o; o += align256((size_t)L->n_spans * D * sizeof(double));
  L->off_block_head = o; o += align256((size_t)L->n_span_blocks * D * sizeof(double));
  L->off_span_flags = o; o += align256((size_t)L->n_spans * sizeof(u32));
  L->off_span_rows = o; o += align256((size_t)L->n_spans * sizeof(u32));
  L->total = std::max<size_t>(o, 256);
}

inline u32 lanes_per_row(u32 D) {
  u32 v = D / 4, p = 1;
  while (p < v) p <<= 1;
  return p;  // 1..64
}

inline u32 blocks_for(u64 threads) { return (u32)((threads + BLOCK - 1) / BLOCK); }

}  // namespace

// Device memory of the entry point that allocates nothing (ctr_lookup_pool_noalloc): a fixed array inside
// the code object, one copy per GPU that loads the library, alive until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; the address kernels can use is looked up once per
// device (with that device current) and kept here.
static __device__ __align__(256) unsigned char scratch[CTR_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[MAX_DEVICES] = {};

// The current device's copy of `scratch`.  The first call on a device asks the runtime for the address;
// later calls (also under stream capture) only read the cached pointer.
int scratch_of_current_device(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return CTR_E_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CTR_E_DEVICE;
    g_scratch_ptr[dev] = (char*)p;
  }
  *out = g_scratch_ptr[dev];
  return CTR_OK;
}

}  // namespace

struct ctr_batch {
  ctr_table* t;
  u64 generation;
  u32 replica, n_keys, n_seg;
  char* ws;
  WorkLayout wl;
  u32* sorted_rows;
  u32* sorted_segs;
};

struct ctr_table {
  ctr_config cfg;
  TableLayout tl;
  u32 D, W, lpr, row_bits, rf;  // rf: floats per row
  u64 R;
  char* mem;
  DevHeader* hdr;
  Slot* slots;
  u64* row_key;
  u32* row_state;
  float* values;
  float* vhat;
  u64 seed_mul;
  float init_scale;
  u64 generation;
  // At most one batch is live per table: it is kept here, and the handle the caller holds is its
  // generation number (never reused), so a stale handle can never be mistaken for a live one.
  ctr_batch cur;
  bool has_live;
  u32 force_span, force_items;  // test hook: 0 = geometry by batch size
  u32 push_windows, push_split;  // execution order of the push's spans (ctr_debug_set_push_order)
  u64 push_order_min_grad_bytes;
  bool profile;
  // stage timers: one (start, stop) event pair per recorded execution since the last read
  std::vector<hipEvent_t> ev_start[CTR_N_STAGES], ev_stop[CTR_N_STAGES];
  size_t ev_used[CTR_N_STAGES];
};

namespace {

struct StageTimer {
  ctr_table* t;
  int stage;
  hipStream_t st;
  bool on;
  size_t idx;
  StageTimer(ctr_table* t_, int stage_, hipStream_t st_) : t(t_), stage(stage_), st(st_), on(false), idx(0) {
    if (!t->profile) return;
    idx = t->ev_used[stage];
    if (idx == t->ev_start[stage].size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return;
      }
      try {
        t->ev_start[stage].push_back(a);
        t->ev_stop[stage].push_back(b);
      } catch (...) {  // no timing for this execution; the lists stay of equal length
        if (t->ev_start[stage].size() > t->ev_stop[stage].size()) t->ev_start[stage].pop_back();
        (void)hipEventDestroy(a);
        (void)hipEventDestroy(b);
        return;
      }
    }
    on = hipEventRecord(t->ev_start[stage][idx], st) == hipSuccess;
  }
  ~StageTimer() {
    if (on && hipEventRecord(t->ev_stop[stage][idx], st) == hipSuccess) t->ev_used[stage] = idx + 1;
  }
};

#define LPR_DISPATCH(lpr, KERNEL, grid, stream, ...)                                                     \
  switch (lpr) {                                                                                         \
    case 1: hipLaunchKernelGGL((KERNEL<1>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;     \
    case 2: hipLaunchKernelGGL((KERNEL<2>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;     \
    case 4: hipLaunchKernelGGL((KERNEL<4>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;     \
    case 8: hipLaunchKernelGGL((KERNEL<8>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;     \
    case 16: hipLaunchKernelGGL((KERNEL<16>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;   \
    case 32: hipLaunchKernelGGL((KERNEL<32>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;   \
    default: hipLaunchKernelGGL((KERNEL<64>), dim3(grid), dim3(BLOCK), 0, stream, __VA_ARGS__); break;   \
  }

inline int launch_status() { return hipGetLastError() == hipSuccess ? CTR_OK : CTR_E_DEVICE; }

// The batch a caller's handle stands for, or null if it is not the table's live one.
inline ctr_batch* live_batch(ctr_table* t, const ctr_batch* handle) {
  return (t->has_live && (uintptr_t)handle == (uintptr_t)t->cur.generation) ? &t->cur : nullptr;
}

int status_code_from_bits(u32 bits) {
  if (bits & ST_INVAL) return CTR_E_INVAL;
  if (bits & ST_BADKEY) return CTR_E_BADKEY;
  if (bits & ST_FULL) return CTR_E_FULL;
  return CTR_OK;
}

}  // namespace

// Key -> row for every occurrence, inserting unseen keys (rows numbered by first occurrence, state
// initialised); on return of the enqueued work occ_row[p] holds the row of keys[p], or the pull has
// failed and was rolled back (device status set).  d_offsets may be null (nothing to validate).
// init_new_rows = false: the caller overwrites the state of every row of the batch anyway (a working-set load).
static void enqueue_lookup_insert(ctr_table* t, const WorkLayout& wl, char* ws, const u64* d_keys, u32 n,
                                  const u32* d_offsets, u32 n_segments, bool init_new_rows, hipStream_t st) {
  u32* occ_row = (u32*)(ws + wl.off_occ_row);
  u32* tile_count = (u32*)(ws + wl.off_tile_count);
  u32* first_bits = (u32*)(ws + wl.off_first_bits);
  u32* pend_list = (u32*)(ws + wl.off_pend_list);
  u32* tile_pending = (u32*)(ws + wl.off_tile_pending);
  const u32 slot_mask = (u32)(t->tl.n_slots - 1);
  {
    StageTimer tm(t, CTR_STAGE_PROBE, st);
    const u64 work = std::max<u64>(n, d_offsets ? (u64)n_segments + 1 : 1);
    const u32 grid = (u32)((work + wl.probe_tile - 1) / wl.probe_tile);  // >= n_probe_tiles
    hipLaunchKernelGGL(k_probe_insert, dim3(grid), dim3(BLOCK), 0, st, t->hdr, t->slots, slot_mask, d_keys, n,
                       d_offsets, n_segments, occ_row, first_bits, pend_list, tile_pending, wl.probe_items);
  }
  {
    StageTimer tm(t, CTR_STAGE_INSERT, st);
    if (n > 0) {
      hipLaunchKernelGGL(k_flag_first, dim3(wl.n_probe_tiles), dim3(BLOCK), 0, st, t->hdr, t->slots, occ_row,
                         pend_list, tile_pending, wl.probe_tile, first_bits);
      hipLaunchKernelGGL(k_count_first, dim3(wl.n_bit_tiles), dim3(BLOCK), 0, st, t->hdr, first_bits,
                         wl.n_bit_words, tile_count);
    }
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(BLOCK), 0, st, t->hdr, tile_count, wl.n_bit_tiles, t->R);
    if (n > 0) {
      hipLaunchKernelGGL(k_assign_rows, dim3(wl.n_bit_tiles), dim3(BLOCK), 0, st, t->hdr, t->slots, occ_row,
                         first_bits, wl.n_bit_words, tile_count, t->row_key);
      if (init_new_rows) {
        const u32 grid = std::min<u32>(blocks_for((u64)n * t->lpr), 4096);
        LPR_DISPATCH(t->lpr, k_init_rows, grid, st, t->hdr, t->row_key, t->values, t->tl.replica_stride, t->W,
                     t->vhat, t->D, t->rf, t->seed_mul, t->init_scale,
                     (t->cfg.flags & CTR_F_BIAS_CORRECTION) ? 0.0f : t->cfg.eps);
      }
      hipLaunchKernelGGL(k_resolve, dim3(wl.n_probe_tiles), dim3(BLOCK), 0, st, t->hdr, t->slots, occ_row,
                         pend_list, tile_pending, wl.probe_tile);
    }
  }
}

extern "C" {

size_t ctr_table_bytes(const ctr_config* cfg) {
  TableLayout L;
  return table_layout(cfg, &L) ? L.total : 0;
}

size_t ctr_workspace_bytes(const ctr_config* cfg, uint64_t max_keys, uint32_t max_segments) {
  (void)max_segments;
  if (!config_ok(cfg) || max_keys >= (1ull << 31)) return 0;
  // The work geometry (span length, probe tile) is chosen from the size of each batch, and a batch just
  // below a threshold needs more span partials than one just above it: the answer covers every batch of
  // at most max_keys occurrences, i.e. the largest layout over max_keys itself and the last size of
  // every geometry class below it (inside a class the layout only grows with the size).
  WorkLayout L;
  work_layout(cfg->dim, max_keys, &L);
  size_t need = L.total;
  for (u64 threshold : {(u64)2 << 20, (u64)4 << 20, (u64)8 << 20}) {
    if (threshold - 1 < max_keys) {
      work_layout(cfg->dim, threshold - 1, &L);
      need = std::max(need, L.total);
    }
  }
  return need;
}

int ctr_table_create(const ctr_config* cfg, void* d_mem, size_t bytes, void* hip_stream, ctr_table** out) {
  if (!cfg || !d_mem || !out) return CTR_E_INVAL;
  TableLayout L;
  if (!table_layout(cfg, &L)) return CTR_E_INVAL;
  if (((uintptr_t)d_mem & 255) != 0) return CTR_E_INVAL;
  if (bytes < L.total) return CTR_E_NOMEM;
  {  // set-up is the place to learn the address of the fixed scratch on this device (ctr_lookup_pool_noalloc)
    char* unused = nullptr;
    if (scratch_of_current_device(&unused) != CTR_OK) return CTR_E_DEVICE;
  }
  ctr_table* t = new (std::nothrow) ctr_table();
  if (!t) return CTR_E_NOMEM;
  t->cfg = *cfg;
  if (t->cfg.load_factor == 0.0f) t->cfg.load_factor = 0.5f;
  t->tl = L;
  t->D = cfg->dim;
  t->W = cfg->n_replicas;
  t->R = cfg->capacity_rows;
  t->lpr = lanes_per_row(t->D);
  t->rf = ((cfg->flags & CTR_F_ADAGRAD) ? 2u : 3u) * t->D;
  t->row_bits = 1;
  while ((1ull << t->row_bits) < t->R) ++t->row_bits;
  t->mem = (char*)d_mem;
  t->hdr = (DevHeader*)(t->mem + L.off_hdr);
  t->slots = (Slot*)(t->mem + L.off_slots);
  t->row_key = (u64*)(t->mem + L.off_row_key);
  t->row_state = (u32*)(t->mem + L.off_row_state);
  t->values = (float*)(t->mem + L.off_values);
  t->vhat = ((cfg->flags & CTR_F_KSTEP) && !(cfg->flags & CTR_F_KSTEP_PROSE)) ? (float*)(t->mem + L.off_vhat) : nullptr;
  t->seed_mul = cfg->init_seed * 0x9E3779B97F4A7C15ull;
  t->init_scale = (float)((double)cfg->init_std / 37837.2);
  t->generation = 0;
  t->has_live = false;
  t->force_span = t->force_items = 0;
  t->push_windows = CTR_PUSH_WINDOWS;
  t->push_split = CTR_PUSH_SPLIT;
  t->push_order_min_grad_bytes = CTR_PUSH_ORDER_MIN_GRAD_BYTES;
  t->profile = false;
  for (int i = 0; i < CTR_N_STAGES; ++i) t->ev_used[i] = 0;
  hipStream_t st = (hipStream_t)hip_stream;
  const u64 work = std::max<u64>(L.n_slots, t->R);
  const u32 grid = (u32)std::min<u64>((work + BLOCK - 1) / BLOCK, 8192);
  hipLaunchKernelGGL(k_table_clear, dim3(grid), dim3(BLOCK), 0, st, t->hdr, t->slots, L.n_slots, t->row_state,
                     t->R, 0u);
  if (launch_status() != CTR_OK) {
    delete t;
    return CTR_E_DEVICE;
  }
  *out = t;
  return CTR_OK;
}

int ctr_table_destroy(ctr_table* t) {
  if (!t) return CTR_E_INVAL;
  for (int i = 0; i < CTR_N_STAGES; ++i) {
    for (hipEvent_t e : t->ev_start[i]) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->ev_stop[i]) (void)hipEventDestroy(e);
  }
  delete t;
  return CTR_OK;
}

static int pull_pool_impl(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                          const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled, bf16_t* d_pooled_bf16,
                          void* d_workspace, size_t workspace_bytes, ctr_batch** batch_out, void* hip_stream) {
  if (!t || !batch_out || !d_offsets || !d_workspace) return CTR_E_INVAL;
  if (replica >= t->W) return CTR_E_INVAL;
  if (n_keys >= (1ull << 31) || n_segments == 0xFFFFFFFFu) return CTR_E_INVAL;
  if (n_keys > 0 && !d_keys) return CTR_E_INVAL;
  if (n_segments > 0 && !d_pooled && !d_pooled_bf16) return CTR_E_INVAL;
  if (((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WorkLayout wl;
  work_layout(t->D, n_keys, &wl, t->force_span, t->force_items);
  if (workspace_bytes < wl.total) return CTR_E_NOMEM;

  t->has_live = false;  // an unpushed batch goes stale
  ctr_batch* b = &t->cur;
  b->t = t;
  b->generation = ++t->generation;
  b->replica = replica;
  b->n_keys = (u32)n_keys;
  b->n_seg = n_segments;
  b->ws = (char*)d_workspace;
  b->wl = wl;
  b->sorted_rows = nullptr;
  b->sorted_segs = nullptr;

  hipStream_t st = (hipStream_t)hip_stream;
  const u32 n = (u32)n_keys;
  u32* occ_row = (u32*)(b->ws + wl.off_occ_row);
  u32* seg_of = (u32*)(b->ws + wl.off_seg_of);
  enqueue_lookup_insert(t, wl, b->ws, (const u64*)d_keys, n, d_offsets, n_segments, true, st);
  if (n_segments > 0) {
    StageTimer tm(t, CTR_STAGE_POOL, st);
    const float* vals = t->values + (u64)replica * t->tl.replica_stride;
    const u32 segs_per_block = (BLOCK / t->lpr) * POOL_NS * POOL_ROUNDS;
    const u32 pgrid = (n_segments + segs_per_block - 1) / segs_per_block;
#define CTR_POOL_LAUNCH(KERNEL) \
  LPR_DISPATCH(t->lpr, KERNEL, pgrid, st, t->hdr, occ_row, seg_of, d_offsets, n_segments, vals, t->D, t->rf, d_pooled, d_pooled_bf16)
    if (d_pooled && d_pooled_bf16) {
      CTR_POOL_LAUNCH(k_pool_both);
    } else if (d_pooled_bf16) {
      CTR_POOL_LAUNCH(k_pool_bf16);
    } else {
      CTR_POOL_LAUNCH(k_pool);
    }
#undef CTR_POOL_LAUNCH
  }
  if (n > 0) {
    StageTimer tm(t, CTR_STAGE_SORT, st);
    u32* hist = (u32*)(b->ws + wl.off_hist);
    u32* digit_total = (u32*)(b->ws + wl.off_digit_total);
    u32* ka = (u32*)(b->ws + wl.off_ka);
    u32* va = (u32*)(b->ws + wl.off_va);
    u32* kb = (u32*)(b->ws + wl.off_kb);
    u32* vb = (u32*)(b->ws + wl.off_vb);
    const u32 passes = (t->row_bits + 7) / 8;
    const u32* kin = occ_row;
    const u32* vin = seg_of;
    u32 shift = 0;
    for (u32 p = 0; p < passes; ++p) {
      // spread the row bits evenly over the passes
      const u32 bits = (t->row_bits - shift + (passes - p) - 1) / (passes - p);
      const u32 mask = (1u << bits) - 1u;
      u32* kout = (p & 1) ? kb : ka;
      u32* vout = (p & 1) ? vb : va;
      hipLaunchKernelGGL(k_sort_hist, dim3(wl.geo.n_chunks), dim3(BLOCK), 0, st, t->hdr, kin, wl.geo, shift, mask,
                         hist);
      hipLaunchKernelGGL(k_sort_scan, dim3(RADIX), dim3(BLOCK), 0, st, t->hdr, hist, wl.geo.n_chunks, digit_total);
      hipLaunchKernelGGL(k_sort_scatter, dim3(wl.geo.n_chunks), dim3(BLOCK), 0, st, t->hdr, kin, vin, kout, vout,
                         wl.geo, shift, mask, hist, digit_total);
      kin = kout;
      vin = vout;
      shift += bits;
    }
    b->sorted_rows = (u32*)kin;
    b->sorted_segs = (u32*)vin;
  }
  if (launch_status() != CTR_OK) return CTR_E_DEVICE;
  t->has_live = true;
  *batch_out = (ctr_batch*)(uintptr_t)b->generation;
  return CTR_OK;
}

int ctr_pull_pool(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                  const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled, void* d_workspace,
                  size_t workspace_bytes, ctr_batch** batch_out, void* hip_stream) {
  return pull_pool_impl(t, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, nullptr, d_workspace,
                        workspace_bytes, batch_out, hip_stream);
}

int ctr_pull_pool_bf16(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                       const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled, uint16_t* d_pooled_bf16,
                       void* d_workspace, size_t workspace_bytes, ctr_batch** batch_out, void* hip_stream) {
  if (n_segments > 0 && !d_pooled_bf16) return CTR_E_INVAL;
  if (((uintptr_t)d_pooled_bf16 & 7) != 0) return CTR_E_INVAL;
  return pull_pool_impl(t, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16, d_workspace,
                        workspace_bytes, batch_out, hip_stream);
}

// Enqueues the lookup-only pooling with its two per-occurrence lists in the given device arrays.
// `timed`: record the stage timers (they create HIP events on first use, so the entry point that
// must not allocate passes false).
static int lookup_pool_enqueue(ctr_table* t, uint32_t replica, const uint64_t* d_keys, u32 n,
                               const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled, bf16_t* pb,
                               u32* occ_row, u32* seg_of, bool timed, hipStream_t st) {
  const bool profile = t->profile;
  if (!timed) t->profile = false;
  {
    StageTimer tm(t, CTR_STAGE_PROBE, st);
    const u64 work = std::max<u64>(n, (u64)n_segments + 1);
    hipLaunchKernelGGL(k_lookup, dim3(blocks_for(work)), dim3(BLOCK), 0, st, t->hdr, t->slots,
                       (u32)(t->tl.n_slots - 1), (const u64*)d_keys, n, d_offsets, n_segments, occ_row);
    hipLaunchKernelGGL(k_lookup_commit, dim3(1), dim3(WAVE), 0, st, t->hdr);
  }
  if (n_segments > 0) {
    StageTimer tm(t, CTR_STAGE_POOL, st);
    const float* vals = t->values + (u64)replica * t->tl.replica_stride;
    const u32 segs_per_block = (BLOCK / t->lpr) * POOL_NS * POOL_ROUNDS;
    const u32 pgrid = (n_segments + segs_per_block - 1) / segs_per_block;
#define CTR_POOL_LAUNCH(KERNEL) \
  LPR_DISPATCH(t->lpr, KERNEL, pgrid, st, t->hdr, occ_row, seg_of, d_offsets, n_segments, vals, t->D, t->rf, d_pooled, pb)
    if (d_pooled && pb) {
      CTR_POOL_LAUNCH(k_pool_lookup_both);
    } else if (pb) {
      CTR_POOL_LAUNCH(k_pool_lookup_bf16);
    } else {
      CTR_POOL_LAUNCH(k_pool_lookup);
    }
#undef CTR_POOL_LAUNCH
  }
  t->profile = profile;
  return launch_status();
}

static int lookup_pool_args_ok(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                               const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                               uint16_t* d_pooled_bf16) {
  if (!t || !d_offsets) return CTR_E_INVAL;
  if (replica >= t->W) return CTR_E_INVAL;
  if (n_keys >= (1ull << 31) || n_segments == 0xFFFFFFFFu) return CTR_E_INVAL;
  if (n_keys > 0 && !d_keys) return CTR_E_INVAL;
  if (n_segments > 0 && !d_pooled && !d_pooled_bf16) return CTR_E_INVAL;
  if (((uintptr_t)d_pooled_bf16 & 7) != 0) return CTR_E_INVAL;
  return CTR_OK;
}

int ctr_lookup_pool(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                    const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled, uint16_t* d_pooled_bf16,
                    void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = lookup_pool_args_ok(t, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16);
  if (rc != CTR_OK) return rc;
  if (!d_workspace || ((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WorkLayout wl;
  work_layout(t->D, n_keys, &wl, t->force_span, t->force_items);
  if (workspace_bytes < wl.total) return CTR_E_NOMEM;
  if (t->has_live && t->cur.ws == (char*)d_workspace) t->has_live = false;  // the live batch's lists are overwritten
  char* ws = (char*)d_workspace;
  return lookup_pool_enqueue(t, replica, d_keys, (u32)n_keys, d_offsets, n_segments, d_pooled,
                             (bf16_t*)d_pooled_bf16, (u32*)(ws + wl.off_occ_row), (u32*)(ws + wl.off_seg_of), true,
                             (hipStream_t)hip_stream);
}

int ctr_lookup_pool_noalloc(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys,
                            const uint32_t* d_offsets, uint32_t n_segments, float* d_pooled,
                            uint16_t* d_pooled_bf16, void* hip_stream) {
  const int rc = lookup_pool_args_ok(t, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16);
  if (rc != CTR_OK) return rc;
  if (n_keys > CTR_NOALLOC_MAX_KEYS) return CTR_E_NOMEM;  // the fixed scratch holds two lists of that many entries
  char* base = nullptr;
  if (scratch_of_current_device(&base) != CTR_OK) return CTR_E_DEVICE;
  // layout of the scratch: occ_row[CTR_NOALLOC_MAX_KEYS] | seg_of[CTR_NOALLOC_MAX_KEYS]; both lists are
  // written in full for the n_keys occurrences of the call before they are read, so nothing needs clearing
  u32* occ_row = (u32*)base;
  u32* seg_of = (u32*)(base + (size_t)CTR_NOALLOC_MAX_KEYS * sizeof(u32));
  return lookup_pool_enqueue(t, replica, d_keys, (u32)n_keys, d_offsets, n_segments, d_pooled,
                             (bf16_t*)d_pooled_bf16, occ_row, seg_of, false, (hipStream_t)hip_stream);
}

// grad_bf16: d_grad_pooled points at bf16 rows instead of fp32 rows
static int push_adam_impl(ctr_table* t, uint32_t replica, ctr_batch* handle, const void* d_grad_pooled, bool grad_bf16,
                          uint32_t mode, void* hip_stream) {
  if (!t || !handle) return CTR_E_INVAL;
  if (replica >= t->W) return CTR_E_INVAL;
  if (mode != CTR_STEP_LOCAL && mode != CTR_STEP_MERGE_PENDING) return CTR_E_INVAL;
  const uint32_t flags = t->cfg.flags;
  const bool kstep = (flags & CTR_F_KSTEP) != 0;
  const bool prose = (flags & CTR_F_KSTEP_PROSE) != 0;
  if ((!kstep || prose) && mode != CTR_STEP_LOCAL) return CTR_E_INVAL;  // only Algorithm 2 as printed defers a step
  ctr_batch* batch = live_batch(t, handle);
  if (!batch) return CTR_E_STATE;  // stale, foreign or already consumed
  if (batch->replica != replica) return CTR_E_STATE;
  if (batch->n_seg > 0 && !d_grad_pooled) return CTR_E_INVAL;

  hipStream_t st = (hipStream_t)hip_stream;
  const WorkLayout& wl = batch->wl;
  const u32 n = batch->n_keys;
  if (flags & CTR_F_BIAS_CORRECTION)  // the step count lives on the device: an empty batch counts, a refused one does not
    hipLaunchKernelGGL(k_push_begin, dim3(1), dim3(WAVE), 0, st, t->hdr, (double)t->cfg.beta1, (double)t->cfg.beta2);
  if (n > 0) {
    AdamParams P;
    P.b1 = (double)t->cfg.beta1;
    P.omb1 = 1.0 - P.b1;
    P.b2 = (double)t->cfg.beta2;
    P.omb2 = 1.0 - P.b2;
    P.eps = (double)t->cfg.eps;
    P.bc1 = P.bc2 = 1.0;  // the bias-corrected update reads its factors from the device header
    P.lr = t->cfg.lr;
    P.kstep = kstep ? 1u : 0u;
    P.mode = (mode == CTR_STEP_MERGE_PENDING) ? 2u : 0u;
    P.pend_bit = (P.mode == 2u) ? (1u << replica) : 0u;
    int kind = STEP_ADAM_OWN;
    if (flags & CTR_F_ADAGRAD) kind = STEP_ADAGRAD;
    else if (flags & CTR_F_BIAS_CORRECTION) kind = STEP_ADAM_KINGMA;
    else if (kstep && !prose && mode == CTR_STEP_LOCAL) kind = STEP_ADAM_SHARED;
    float* vals = t->values + (u64)replica * t->tl.replica_stride;
    double* head = (double*)(batch->ws + wl.off_head);
    double* tail = (double*)(batch->ws + wl.off_tail);
    double* block_head = (double*)(batch->ws + wl.off_block_head);
    u32* span_flags = (u32*)(batch->ws + wl.off_span_flags);
    u32* span_rows = (u32*)(batch->ws + wl.off_span_rows);
#define CTR_SPAN_LAUNCH(KERNEL)                                                                                   \
  LPR_DISPATCH(t->lpr, KERNEL, grid, st, t->hdr, batch->sorted_rows, batch->sorted_segs, n, wl.span, d_grad_pooled, \
               vals, t->vhat, t->row_state, t->D, t->rf, P, head, tail, span_flags, span_rows, order, cold_count)
#define CTR_FIXUP_LAUNCH(KERNEL)                                                                                 \
  LPR_DISPATCH(t->lpr, KERNEL, fgrid, st, t->hdr, batch->sorted_rows, n, wl.n_spans, wl.span, vals, t->vhat,       \
               t->row_state, t->D, t->rf, P, head, tail, block_head, span_flags)
    const u32 grid = blocks_for((u64)wl.n_spans * t->lpr);
    const u32 *order = nullptr, *cold_count = nullptr;
    bool hot_launch = false;
    // Execution order of the spans: one pass of the radix sort over (window key, span index).  Its four
    // short arrays live in the sort's key buffer that does not hold the sorted list.
    if (t->push_windows) {
      u32* ka = (u32*)(batch->ws + wl.off_ka);
      u32* kb = (u32*)(batch->ws + wl.off_kb);
      u32* spare = (batch->sorted_rows == ka) ? kb : ka;
      const u32 ns4 = (wl.n_spans + 3u) & ~3u;  // the sort reads 16 bytes at a time
      const u64 grad_bytes = (u64)batch->n_seg * t->D * (grad_bf16 ? 2u : 4u);
      if (grad_bytes >= t->push_order_min_grad_bytes && batch->n_seg > 0 && 16ull * ns4 <= 4ull * n) {
        StageTimer tm(t, CTR_STAGE_ORDER, st);
        u32 *key_in = spare, *val_in = spare + ns4, *key_out = spare + 2 * ns4, *val_out = spare + 3 * ns4;
        u32 seg_shift = 0;
        while (((batch->n_seg - 1) >> seg_shift) >= t->push_windows) ++seg_shift;
        const SortGeom g2 = sort_geom(wl.n_spans);
        u32* hist = (u32*)(batch->ws + wl.off_hist);
        u32* digit_total = (u32*)(batch->ws + wl.off_digit_total);
        hipLaunchKernelGGL(k_span_keys, dim3(blocks_for(wl.n_spans)), dim3(BLOCK), 0, st, t->hdr, batch->sorted_rows,
                           batch->sorted_segs, n, wl.span, wl.n_spans, seg_shift, t->push_windows,
                           t->push_split == 2u ? 1u : 0u, key_in, val_in);
        hipLaunchKernelGGL(k_sort_hist, dim3(g2.n_chunks), dim3(BLOCK), 0, st, t->hdr, key_in, g2, 0u, 255u, hist);
        hipLaunchKernelGGL(k_sort_scan, dim3(RADIX), dim3(BLOCK), 0, st, t->hdr, hist, g2.n_chunks, digit_total);
        hipLaunchKernelGGL(k_sort_scatter, dim3(g2.n_chunks), dim3(BLOCK), 0, st, t->hdr, key_in, val_in, key_out,
                           val_out, g2, 0u, 255u, hist, digit_total);
        order = val_out;
        if (t->push_split == 1u) {
          cold_count = digit_total + t->push_windows;  // spans with the key one past the last window
          hot_launch = true;
        }
      }
    }
    {
      StageTimer tm(t, CTR_STAGE_PUSH, st);
      if (hot_launch) {
        if (grad_bf16) {
          LPR_DISPATCH(t->lpr, k_push_hot_g16, grid, st, t->hdr, batch->sorted_rows, batch->sorted_segs, n, wl.span,
                       d_grad_pooled, t->D, head, tail, span_flags, span_rows, order, cold_count);
        } else {
          LPR_DISPATCH(t->lpr, k_push_hot, grid, st, t->hdr, batch->sorted_rows, batch->sorted_segs, n, wl.span,
                       d_grad_pooled, t->D, head, tail, span_flags, span_rows, order, cold_count);
        }
      }
      if (grad_bf16) {
        switch (kind) {
          case STEP_ADAM_SHARED: CTR_SPAN_LAUNCH(k_push_span_shared_g16); break;
          case STEP_ADAGRAD: CTR_SPAN_LAUNCH(k_push_span_adagrad_g16); break;
          case STEP_ADAM_KINGMA: CTR_SPAN_LAUNCH(k_push_span_kingma_g16); break;
          default: CTR_SPAN_LAUNCH(k_push_span_g16); break;
        }
      } else {
        switch (kind) {
          case STEP_ADAM_SHARED: CTR_SPAN_LAUNCH(k_push_span_shared); break;
          case STEP_ADAGRAD: CTR_SPAN_LAUNCH(k_push_span_adagrad); break;
          case STEP_ADAM_KINGMA: CTR_SPAN_LAUNCH(k_push_span_kingma); break;
          default: CTR_SPAN_LAUNCH(k_push_span); break;
        }
      }
    }
    {
      StageTimer tm(t, CTR_STAGE_FIXUP, st);
      LPR_DISPATCH(t->lpr, k_push_block_heads, blocks_for((u64)wl.n_span_blocks * WAVE), st, t->hdr,
                   batch->sorted_rows, wl.n_spans, wl.span, t->D, head, block_head, span_flags);
      const u32 fgrid = blocks_for((u64)wl.n_spans * WAVE);
      switch (kind) {
        case STEP_ADAM_SHARED: CTR_FIXUP_LAUNCH(k_push_fixup_shared); break;
        case STEP_ADAGRAD: CTR_FIXUP_LAUNCH(k_push_fixup_adagrad); break;
        case STEP_ADAM_KINGMA: CTR_FIXUP_LAUNCH(k_push_fixup_kingma); break;
        default: CTR_FIXUP_LAUNCH(k_push_fixup); break;
      }
      const u32 grid = std::min<u32>(blocks_for(wl.n_spans), 128);
      hipLaunchKernelGGL(k_count_unique, dim3(grid), dim3(BLOCK), 0, st, t->hdr, span_rows, wl.n_spans);
    }
#undef CTR_SPAN_LAUNCH
#undef CTR_FIXUP_LAUNCH
  }
  t->has_live = false;
  return launch_status();
}

int ctr_push_adam(ctr_table* t, uint32_t replica, ctr_batch* handle, const float* d_grad_pooled, uint32_t mode,
                  void* hip_stream) {
  return push_adam_impl(t, replica, handle, d_grad_pooled, false, mode, hip_stream);
}

int ctr_push_adam_bf16(ctr_table* t, uint32_t replica, ctr_batch* handle, const uint16_t* d_grad_pooled_bf16,
                       uint32_t mode, void* hip_stream) {
  if (((uintptr_t)d_grad_pooled_bf16 & 7) != 0) return CTR_E_INVAL;
  return push_adam_impl(t, replica, handle, d_grad_pooled_bf16, true, mode, hip_stream);
}

int ctr_kstep_merge(ctr_table* t, void* hip_stream) {
  if (!t) return CTR_E_INVAL;
  if (!(t->cfg.flags & CTR_F_KSTEP)) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  StageTimer tm(t, CTR_STAGE_MERGE, st);
  const u32 grid = std::min<u32>(blocks_for(t->R * t->lpr), 16384);
  if (t->cfg.flags & CTR_F_KSTEP_PROSE) {
    LPR_DISPATCH(t->lpr, k_merge_prose, grid, st, t->hdr, t->values, t->tl.replica_stride, t->W, t->vhat,
                 t->row_state, t->D, t->cfg.lr);
  } else {
    LPR_DISPATCH(t->lpr, k_merge, grid, st, t->hdr, t->values, t->tl.replica_stride, t->W, t->vhat, t->row_state,
                 t->D, t->cfg.lr);
  }
  return launch_status();
}

int ctr_table_load(ctr_table* t, const uint64_t* d_keys, uint64_t n_keys, const float* d_x, const float* d_m,
                   const float* d_v, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!t || !d_workspace) return CTR_E_INVAL;
  if (n_keys >= (1ull << 31)) return CTR_E_INVAL;
  const bool has_m = !(t->cfg.flags & CTR_F_ADAGRAD);
  if (n_keys > 0 && (!d_keys || !d_x || !d_v || (has_m && !d_m))) return CTR_E_INVAL;
  if (((uintptr_t)d_workspace & 255) != 0) return CTR_E_INVAL;
  WorkLayout wl;
  work_layout(t->D, n_keys, &wl, t->force_span, t->force_items);
  if (workspace_bytes < wl.total) return CTR_E_NOMEM;
  t->has_live = false;  // the workspace of an unpushed batch may be this one: it goes stale
  ++t->generation;
  hipStream_t st = (hipStream_t)hip_stream;
  const u32 n = (u32)n_keys;
  enqueue_lookup_insert(t, wl, (char*)d_workspace, (const u64*)d_keys, n, nullptr, 0, false, st);
  if (n > 0) {
    const u32* occ_row = (const u32*)((char*)d_workspace + wl.off_occ_row);
    LPR_DISPATCH(t->lpr, k_load_rows, blocks_for((u64)n * t->lpr), st, t->hdr, occ_row, n, t->values,
                 t->tl.replica_stride, t->W, t->vhat, t->D, t->rf, d_x, d_m, d_v);
  }
  return launch_status();
}

int ctr_table_clear(ctr_table* t, void* hip_stream) {
  if (!t) return CTR_E_INVAL;
  t->has_live = false;
  ++t->generation;
  hipStream_t st = (hipStream_t)hip_stream;
  const u64 work = std::max<u64>(t->tl.n_slots, t->R);
  const u32 grid = (u32)std::min<u64>((work + BLOCK - 1) / BLOCK, 8192);
  hipLaunchKernelGGL(k_table_clear, dim3(grid), dim3(BLOCK), 0, st, t->hdr, t->slots, t->tl.n_slots, t->row_state,
                     t->R, 1u);
  return launch_status();
}

int ctr_table_collect(ctr_table* t, uint32_t replica, const uint64_t* d_keys, uint64_t n_keys, float* d_x,
                      float* d_m, float* d_v, uint32_t* d_found, void* hip_stream) {
  if (!t || replica >= t->W) return CTR_E_INVAL;
  if (n_keys >= (1ull << 31)) return CTR_E_INVAL;
  if (n_keys > 0 && !d_keys) return CTR_E_INVAL;
  if (d_m && (t->cfg.flags & CTR_F_ADAGRAD)) return CTR_E_INVAL;
  if (n_keys == 0) return CTR_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const float* vals = t->values + (u64)replica * t->tl.replica_stride;
  LPR_DISPATCH(t->lpr, k_collect_rows, blocks_for(n_keys * t->lpr), st, t->hdr, t->slots,
               (u32)(t->tl.n_slots - 1), (const u64*)d_keys, (u32)n_keys, vals, t->D, t->rf, d_x, d_m, d_v, d_found);
  return launch_status();
}

int ctr_table_size(ctr_table* t, uint64_t* n_rows, void* hip_stream) {
  if (!t || !n_rows) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  DevHeader h;
  if (hipMemcpyAsync(&h, t->hdr, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  *n_rows = h.n_rows;
  return CTR_OK;
}

int ctr_table_export(ctr_table* t, uint32_t replica, uint64_t* h_keys, float* h_x, float* h_m, float* h_v,
                     float* h_vhat, void* hip_stream) {
  if (!t || replica >= t->W) return CTR_E_INVAL;
  if (h_vhat && !t->vhat) return CTR_E_INVAL;
  const bool adagrad = (t->cfg.flags & CTR_F_ADAGRAD) != 0;
  if (h_m && adagrad) return CTR_E_INVAL;  // AdaGrad rows have no first moment
  hipStream_t st = (hipStream_t)hip_stream;
  uint64_t n = 0;
  int rc = ctr_table_size(t, &n, hip_stream);
  if (rc != CTR_OK) return rc;
  if (n == 0) return CTR_OK;
  const size_t D = t->D, rowb = D * sizeof(float), pitch = (size_t)t->rf * sizeof(float);
  const float* vals = t->values + (u64)replica * t->tl.replica_stride;
  bool ok = true;
  if (h_keys) ok = ok && hipMemcpyAsync(h_keys, t->row_key, n * sizeof(u64), hipMemcpyDeviceToHost, st) == hipSuccess;
  if (h_vhat) ok = ok && hipMemcpyAsync(h_vhat, t->vhat, n * rowb, hipMemcpyDeviceToHost, st) == hipSuccess;
  // Rows are [x | m | v] interleaved: whole rows come over in contiguous chunks and are split on
  // the host (a strided device copy of 64..1024-byte pieces is far slower than that).
  struct Field { float* dst; size_t off; };
  const Field fields[3] = {{h_x, 0}, {h_m, D}, {h_v, adagrad ? D : 2 * D}};
  if (h_x || h_m || h_v) {
    const size_t chunk_rows = std::max<size_t>(1, ((size_t)32 << 20) / pitch);
    std::vector<float> tmp;
    try {
      tmp.resize(std::min<size_t>(chunk_rows, n) * t->rf);
    } catch (const std::bad_alloc&) {
      return CTR_E_NOMEM;
    }
    for (size_t r0 = 0; r0 < n && ok; r0 += chunk_rows) {
      const size_t cnt = std::min<size_t>(chunk_rows, n - r0);
      ok = ok && hipMemcpyAsync(tmp.data(), vals + r0 * t->rf, cnt * pitch, hipMemcpyDeviceToHost, st) == hipSuccess;
      ok = ok && hipStreamSynchronize(st) == hipSuccess;
      if (!ok) break;
      for (const Field& f : fields) {
        if (!f.dst) continue;
        for (size_t r = 0; r < cnt; ++r) memcpy(f.dst + (r0 + r) * D, tmp.data() + r * t->rf + f.off, rowb);
      }
    }
  }
  ok = ok && hipStreamSynchronize(st) == hipSuccess;
  return ok ? CTR_OK : CTR_E_DEVICE;
}

int ctr_batch_export(ctr_table* t, ctr_batch* handle, uint64_t* n_unique, uint64_t* h_uniq, uint32_t* h_rows,
                     uint32_t* h_inverse, void* hip_stream) {
  if (!t || !handle) return CTR_E_INVAL;
  const ctr_batch* batch = live_batch(t, handle);
  if (!batch) return CTR_E_STATE;
  hipStream_t st = (hipStream_t)hip_stream;
  DevHeader h;
  if (hipMemcpyAsync(&h, t->hdr, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  if (h.status) return CTR_E_STATE;  // the pull failed: there is no dedup result
  const size_t n = batch->n_keys;
  // Re-expression of device results for comparison: the device keeps the batch's
  // distinct set as row ids; the canonical form lists the keys in ascending order.
  try {  // host containers below: no exception may cross the C boundary
    std::vector<u32> occ(n);
    std::vector<u64> row_key(h.n_rows);
    if (n && hipMemcpyAsync(occ.data(), batch->ws + batch->wl.off_occ_row, n * sizeof(u32), hipMemcpyDeviceToHost,
                            st) != hipSuccess)
      return CTR_E_DEVICE;
    if (h.n_rows && hipMemcpyAsync(row_key.data(), t->row_key, (size_t)h.n_rows * sizeof(u64),
                                   hipMemcpyDeviceToHost, st) != hipSuccess)
      return CTR_E_DEVICE;
    if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
    std::vector<u32> rows(occ);
    std::sort(rows.begin(), rows.end());
    rows.erase(std::unique(rows.begin(), rows.end()), rows.end());
    for (u32 r : rows)
      if (r >= h.n_rows) return CTR_E_DEVICE;
    std::vector<std::pair<u64, u32>> kr(rows.size());
    for (size_t i = 0; i < rows.size(); ++i) kr[i] = {row_key[rows[i]], rows[i]};
    std::sort(kr.begin(), kr.end());
    if (n_unique) *n_unique = kr.size();
    if (h_uniq)
      for (size_t i = 0; i < kr.size(); ++i) h_uniq[i] = kr[i].first;
    if (h_rows)
      for (size_t i = 0; i < kr.size(); ++i) h_rows[i] = kr[i].second;
    if (h_inverse) {
      std::vector<u32> index_of_row(h.n_rows, 0);
      for (size_t i = 0; i < kr.size(); ++i) index_of_row[kr[i].second] = (u32)i;
      for (size_t p = 0; p < n; ++p) h_inverse[p] = index_of_row[occ[p]];
    }
  } catch (const std::bad_alloc&) {
    return CTR_E_NOMEM;
  }
  return CTR_OK;
}

int ctr_batch_stats(ctr_table* t, uint64_t* n_unique, uint64_t* n_new, void* hip_stream) {
  if (!t) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  DevHeader h;
  if (hipMemcpyAsync(&h, t->hdr, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  if (n_unique) *n_unique = h.n_unique;
  if (n_new) *n_new = h.n_new;
  return CTR_OK;
}

int ctr_merge_stats(ctr_table* t, uint64_t* rows_merged, uint64_t* pending_applied, void* hip_stream) {
  if (!t || !rows_merged) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  DevHeader h;
  if (hipMemcpyAsync(&h, t->hdr, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  *rows_merged = h.rows_merged;
  if (pending_applied) *pending_applied = h.merge_pending;
  return CTR_OK;
}

int ctr_stream_copy(void* d_dst, const void* d_src, size_t bytes, int non_temporal, void* hip_stream) {
  if (!d_dst || !d_src || bytes == 0 || (bytes & 15) != 0) return CTR_E_INVAL;
  if ((((uintptr_t)d_dst | (uintptr_t)d_src) & 15) != 0) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const u64 n16 = bytes / 16;
  const u32 grid = (u32)std::min<u64>((n16 + BLOCK - 1) / BLOCK, 256 * 16);  // 16 blocks per compute unit
  if (non_temporal)
    hipLaunchKernelGGL(k_stream_copy<true>, dim3(grid), dim3(BLOCK), 0, st, (const vf4*)d_src, (vf4*)d_dst, n16);
  else
    hipLaunchKernelGGL(k_stream_copy<false>, dim3(grid), dim3(BLOCK), 0, st, (const vf4*)d_src, (vf4*)d_dst, n16);
  return launch_status();
}

int ctr_last_status(ctr_table* t, void* hip_stream) {
  if (!t) return CTR_E_INVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  DevHeader h;
  if (hipMemcpyAsync(&h, t->hdr, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  if (h.status == 0) return CTR_OK;
  // clear status, pull_err and rollback (three consecutive words after n_rows)
  if (hipMemsetAsync((char*)t->hdr + offsetof(DevHeader, status), 0, 3 * sizeof(u32), st) != hipSuccess)
    return CTR_E_DEVICE;
  if (hipStreamSynchronize(st) != hipSuccess) return CTR_E_DEVICE;
  return status_code_from_bits(h.status);
}

int ctr_debug_set_geometry(ctr_table* t, uint32_t span, uint32_t probe_items) {
  if (!t) return CTR_E_INVAL;
  if (span != 0 && span != 16 && span != 32 && span != 64 && span != 128) return CTR_E_INVAL;
  if (probe_items != 0 && probe_items != 1 && probe_items != (uint32_t)PROBE_MAX_ITEMS) return CTR_E_INVAL;
  t->force_span = span;
  t->force_items = probe_items;
  return CTR_OK;
}

int ctr_debug_set_push_order(ctr_table* t, uint32_t windows, uint32_t split_launch, uint64_t min_grad_bytes) {
  if (!t) return CTR_E_INVAL;
  if (windows > 128 || (windows & (windows - 1)) != 0 || split_launch > 2) return CTR_E_INVAL;
  t->push_windows = windows;
  t->push_split = split_launch;
  t->push_order_min_grad_bytes = min_grad_bytes;
  return CTR_OK;
}

int ctr_profile_enable(ctr_table* t, int on) {
  if (!t) return CTR_E_INVAL;
  t->profile = on != 0;
  return CTR_OK;
}

int ctr_profile_read(ctr_table* t, float* h_ms, uint32_t* h_count) {
  if (!t || !h_ms) return CTR_E_INVAL;
  if (hipDeviceSynchronize() != hipSuccess) return CTR_E_DEVICE;
  for (int i = 0; i < CTR_N_STAGES; ++i) {
    float total = 0.0f;
    for (size_t k = 0; k < t->ev_used[i]; ++k) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, t->ev_start[i][k], t->ev_stop[i][k]) != hipSuccess) return CTR_E_DEVICE;
      total += ms;
    }
    h_ms[i] = total;
    if (h_count) h_count[i] = (uint32_t)t->ev_used[i];
    t->ev_used[i] = 0;
  }
  return CTR_OK;
}

}  // extern "C"
