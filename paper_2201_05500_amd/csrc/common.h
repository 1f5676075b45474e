// Device-side building blocks shared by the kernels of the sparse embedding cycle (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ctr {

typedef unsigned long long u64;
typedef uint32_t u32;

constexpr int WAVE = 64;
constexpr int BLOCK = 256;  // 4 waves; every kernel here is launched with this block size

// key index
constexpr u64 KEY_EMPTY = ~0ull;           // reserved key: marks a free slot
constexpr u32 ROW_PENDING = 0xFFFFFFFFu;   // slot claimed in this pull, row not assigned yet
constexpr u32 OCC_PEND_FLAG = 0x80000000u; // occ_row entry = flag | slot index, row assigned later
constexpr u32 OCC_INVALID = 0xFFFFFFFFu;   // occurrence whose key could not be placed

// deferred status bits (device header)
constexpr u32 ST_INVAL = 1u, ST_BADKEY = 2u, ST_FULL = 4u;

// per-row state word (k-step mode): bit j = replica j has a pending merge-step update
constexpr u32 RS_TOUCHED = 0x80000000u;

struct __attribute__((aligned(16))) Slot {
  u64 key;
  u32 row;
  u32 first_p;  // smallest occurrence index of the key in the pull that inserted it
};

struct DevHeader {
  u32 n_rows;       // rows in use
  u32 status;       // sticky deferred error bits; kernels are no-ops while it is set
  u32 pull_err;     // errors seen so far by the pull in flight
  u32 rollback;     // 1: the pull in flight failed, its tentative inserts are being undone
  u32 n_rows_base;  // n_rows before the pull in flight
  u32 n_new;        // rows created by the last pull
  u32 n_unique;     // distinct keys of the last pushed batch
  u32 n_push;       // pushes accepted so far: the step count t of the bias-corrected row update
  double bc1, bc2;  // 1 / (1 - beta1^t), 1 / (1 - beta2^t) of the push in flight (bias-corrected form only)
  u64 rows_merged;  // rows averaged by all k-step merges so far (those touched since the merge before)
  u64 merge_pending;  // (row, replica) pairs whose deferred model step those merges applied
  u32 pad[48];
};
constexpr int HDR_WORD_N_PUSH = 7;  // index of n_push among the header's 32-bit words
static_assert(sizeof(DevHeader) == 256, "header is one 256-byte block");

// 64-bit finalizer of MurmurHash3 (public domain): slot choice in the key index.
__device__ __forceinline__ u64 hash_key(u64 h) {
  h ^= h >> 33;
  h *= 0xff51afd7ed558ccdull;
  h ^= h >> 33;
  h *= 0xc4ceb9fe1a85ec53ull;
  h ^= h >> 33;
  return h;
}

// Row initialiser: a counter-based stand-in for a normal draw, defined in
// integer arithmetic so that any implementation reproduces it bit for bit:
// z = splitmix64-finalizer((key ^ seed*GOLDEN) + (d+1)*C); the four 16-bit
// fields of z are summed, centred on 131070 and scaled by one float.
__device__ __forceinline__ float init_value(u64 seed_mul, u64 key, u32 d, float scale) {
  u64 z = (key ^ seed_mul) + (u64)(d + 1) * 0xD1B54A32D192ED03ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  int s = (int)(z & 0xFFFF) + (int)((z >> 16) & 0xFFFF) + (int)((z >> 32) & 0xFFFF) + (int)(z >> 48);
  return (float)(s - 131070) * scale;
}

__device__ __forceinline__ u32 ld_relaxed(const u32* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 ld_relaxed(const u64* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Inclusive scan across the 64 lanes of a wave.
__device__ __forceinline__ u32 wave_inclusive_scan(u32 v) {
  const int lane = lane_id();
#pragma unroll
  for (int off = 1; off < WAVE; off <<= 1) {
    u32 n = __shfl_up(v, off, WAVE);
    if (lane >= off) v += n;
  }
  return v;
}

// Exclusive scan over the 256 threads of a block; `total` receives the block sum.
// `lds` must hold 4 words; the call contains barriers, so every thread must reach it.
__device__ __forceinline__ u32 block_exclusive_scan(u32 v, u32* lds, u32& total) {
  const u32 inc = wave_inclusive_scan(v);
  __syncthreads();  // protects lds reuse across consecutive calls
  if (lane_id() == WAVE - 1) lds[wave_id()] = inc;
  __syncthreads();
  u32 base = 0;
  const u32 w0 = lds[0], w1 = lds[1], w2 = lds[2], w3 = lds[3];
  const int w = wave_id();
  if (w > 0) base += w0;
  if (w > 1) base += w1;
  if (w > 2) base += w2;
  total = w0 + w1 + w2 + w3;
  return base + inc - v;
}

struct __attribute__((aligned(16))) f4 {
  float x, y, z, w;
};
struct d4 {
  double x, y, z, w;
};

__device__ __forceinline__ f4 ldg4(const float* p) { return *reinterpret_cast<const f4*>(p); }
__device__ __forceinline__ void stg4(float* p, f4 v) { *reinterpret_cast<f4*>(p) = v; }

// Streaming variants for data that is used once: the access carries the non-temporal hint, so the
// line is not kept in the caches at the expense of data that will be used again.
typedef float vf4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f4 ldg4_stream(const float* p) {
  const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));
  return f4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ void stg4_stream(float* p, f4 v) {
  __builtin_nontemporal_store(vf4{v.x, v.y, v.z, v.w}, reinterpret_cast<vf4*>(p));
}

// bfloat16 as its 16-bit pattern; rounding from fp32 is nearest-even on the bit pattern.
typedef uint16_t bf16_t;
__device__ __forceinline__ bf16_t to_bf16(float f) {
  const u32 u = __float_as_uint(f);
  return (bf16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float from_bf16(bf16_t h) { return __uint_as_float((u32)h << 16); }
__device__ __forceinline__ void stg4_bf16(bf16_t* p, f4 v) {
  ushort4 o;
  o.x = to_bf16(v.x); o.y = to_bf16(v.y); o.z = to_bf16(v.z); o.w = to_bf16(v.w);
  *reinterpret_cast<ushort4*>(p) = o;
}

}  // namespace ctr
