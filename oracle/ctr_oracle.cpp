// CPU oracle for the per-mini-batch sparse embedding cycle.
//
// THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the plain, slow,
// single-threaded statement of what the cycle computes, written from the
// paper, and exists only so that tests, the smoke check and the benchmark's
// CPU-baseline leg can compare the HIP path against it.  It shares no code,
// header, table or constant generator with the HIP path.
//
// What each function follows:
//   * key -> row map with insert-on-miss: the HBM hash table that holds the
//     working parameters of a batch (Section 2.3; Algorithm 1, the
//     insert_into_hash_table and pull steps).  Here: std::unordered_map.
//   * union of referenced keys: the "identify the union of the referenced
//     parameters" step of the training workflow (Section 2.3).
//   * per-slot sum pooling: the embedding layer of Section 2.1; the paper does
//     not define a pooling rule, the build's problem statement fixes it as a
//     per-(sample, slot) sum with an empty slot giving zeros.
//   * push: the push_parameters_updates_back step of Algorithm 1; one update
//     per distinct key with the sum of the gradients of its occurrences.
//   * Adam arithmetic and the k-step merge: Algorithm 2 (k-step Adam),
//     literally: m_0 = 0, v_0 = eps, no bias correction, no eps in the
//     denominator, a shared denominator v_t frozen between merges, and on a
//     merge step the averaged v is formed first and the k-th model update is
//     applied with it inside the average.
//
// Arithmetic: state (x, m, v, shared v) is stored as IEEE binary32, which is
// the table format the build's configuration fixes.  Every assignment of
// Algorithm 2 and every sum is evaluated in binary64 from the stored values
// and rounded once when stored.  Hyper-parameters arrive as binary32 and are
// promoted.  Compile with -ffp-contract=off.
//
// Readings taken where the paper is silent (also listed in the design notes):
//   * rows not referenced by a push are left untouched (lazy/sparse Adam);
//   * a key occurring c times in a batch takes ONE step with the sum of its c
//     gradients, no division;
//   * new keys get consecutive row ids in order of first occurrence in the
//     batch, x = init(seed, key, d), m = 0, v = shared v = eps (Algorithm 2,
//     "Initialize");
//   * replicas share one key -> row map; a miss by any replica creates the row
//     in all of them with the same init, so a replica that never saw a key
//     enters the merge average holding init(key), m = 0, v = eps;
//   * m is never averaged; local v is never overwritten by the average;
//   * the merge covers rows touched by any replica since the previous merge,
//     and a replica that did not touch a row on the merge step contributes its
//     x with no step term.
//
// Variants (selected at creation; each has its own pins):
//   * AdaGrad, the optimizer the paper uses for sparse parameters (Section 5): rows hold x and an
//     accumulator G; G_0 = eps (placed as Algorithm 2 places it), G += g^2, x -= lr g / sqrt(G).
//   * the prose reading of Section 4 ("standard Adam updates are applied" locally, weights and v
//     averaged every k steps): every step divides by the worker's own v; the merge sets every x
//     to the mean of the x_j and every v_j to the mean of the v_j.
//   * the Adam the paper cites (Kingma & Ba): m_0 = v_0 = 0, bias-corrected moments, eps added to
//     the root, t = number of pushes accepted so far.
//
// Pins (tests/test_oracle_*.py): closed forms of the Adam recurrences for a
// constant gradient, beta1 = 0, duplicate keys == summed gradient, k = 1 with
// one replica == single-table Adam bit for bit, the averaged-iterate and
// consensus identities of the convergence proof (Section 4, proof sketch), the
// linearity of the v recursion, symmetric replicas, brute force over tiny
// inputs with exact rational sums, capacity and sentinel edge cases.
// Not pinned (parity unpinned): the paper's accuracy claims (AUC), which need
// its data and model.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <unordered_set>
#include <vector>

namespace {

enum { ORC_OK = 0, ORC_E_INVAL = 1, ORC_E_NOMEM = 2, ORC_E_FULL = 3, ORC_E_BADKEY = 4,
       ORC_E_STATE = 5 };
enum { STEP_LOCAL = 0, STEP_MERGE_PENDING = 1 };
enum { VAR_ALG2 = 0, VAR_ADAGRAD = 1, VAR_PROSE = 2, VAR_KINGMA = 3 };

const uint64_t SENTINEL = ~0ULL;

struct Table {
  uint64_t R = 0;
  uint32_t D = 0, W = 1;
  float lr = 0, b1 = 0, b2 = 0, eps = 0;
  uint64_t seed = 0;
  float init_std = 0;
  int kstep = 0;
  int variant = VAR_ALG2;
  uint64_t n_push = 0;  // pushes accepted so far (step count of the bias-corrected form)
  uint64_t n_rows = 0;
  std::unordered_map<uint64_t, uint32_t> row_of;
  std::vector<uint64_t> key_of_row;
  std::vector<std::vector<float>> x, m, v;  // [W][n_rows*D]
  std::vector<float> vhat;                  // [n_rows*D], k-step mode only
  std::vector<std::vector<uint8_t>> pending;  // [W][n_rows]
  std::vector<uint8_t> touched;               // [n_rows]
  // result of the last pull
  bool batch_valid = false;
  uint32_t batch_replica = 0;
  std::vector<uint64_t> uniq;
  std::vector<uint32_t> rows, inverse, offsets;
  uint64_t n_new_last = 0;
};

inline uint64_t finalize64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

// Deterministic stand-in for a N(0, init_std^2) draw, specified in integer
// arithmetic: sum of the four 16-bit fields of a 64-bit hash of
// (seed, key, d), centred, times one binary32 constant.
inline float init_value(uint64_t seed, uint64_t key, uint32_t d, float scale) {
  uint64_t z = (key ^ (seed * 0x9E3779B97F4A7C15ULL)) + (uint64_t)(d + 1) * 0xD1B54A32D192ED03ULL;
  z = finalize64(z);
  int s = (int)(z & 0xFFFF) + (int)((z >> 16) & 0xFFFF) + (int)((z >> 32) & 0xFFFF) + (int)(z >> 48);
  return (float)(s - 131070) * scale;
}

inline float init_scale(float init_std) { return (float)((double)init_std / 37837.2); }

}  // namespace

extern "C" {

void* orc_create(uint64_t R, uint32_t D, uint32_t W, float lr, float b1, float b2, float eps,
                 uint64_t seed, float init_std, int kstep, int variant) {
  if (R == 0 || D == 0 || W == 0) return nullptr;
  if (variant < VAR_ALG2 || variant > VAR_KINGMA) return nullptr;
  if (variant == VAR_PROSE && !kstep) return nullptr;
  if ((variant == VAR_ADAGRAD || variant == VAR_KINGMA) && (kstep || W != 1)) return nullptr;
  if (!kstep && W != 1) return nullptr;
  Table* t = new Table();
  t->R = R; t->D = D; t->W = W; t->lr = lr; t->b1 = b1; t->b2 = b2; t->eps = eps;
  t->seed = seed; t->init_std = init_std; t->kstep = kstep; t->variant = variant;
  t->x.resize(W); t->m.resize(W); t->v.resize(W); t->pending.resize(W);
  // address space only; pages are committed as rows are created
  for (uint32_t j = 0; j < W; ++j) {
    t->x[j].reserve((size_t)R * D); t->m[j].reserve((size_t)R * D); t->v[j].reserve((size_t)R * D);
  }
  if (kstep && variant != VAR_PROSE) t->vhat.reserve((size_t)R * D);
  return t;
}

void orc_destroy(void* h) { delete (Table*)h; }

uint64_t orc_n_rows(void* h) { return ((Table*)h)->n_rows; }
uint64_t orc_batch_n_unique(void* h) { return ((Table*)h)->batch_valid ? ((Table*)h)->uniq.size() : 0; }
uint64_t orc_batch_n_new(void* h) { return ((Table*)h)->n_new_last; }

float orc_init_value(uint64_t seed, uint64_t key, uint32_t d, float init_std) {
  return init_value(seed, key, d, init_scale(init_std));
}

// Row id of a key, or -1.
int64_t orc_lookup(void* h, uint64_t key) {
  Table* t = (Table*)h;
  auto it = t->row_of.find(key);
  return it == t->row_of.end() ? -1 : (int64_t)it->second;
}

// Pull: dedup, lookup with insert-on-miss, per-segment sum pooling.
int orc_pull_pool(void* h, uint32_t replica, const uint64_t* keys, uint64_t n_keys,
                  const uint32_t* offsets, uint32_t n_seg, float* pooled) {
  Table* t = (Table*)h;
  const uint32_t D = t->D;
  if (replica >= t->W) return ORC_E_INVAL;
  if (offsets[0] != 0 || offsets[n_seg] != n_keys) return ORC_E_INVAL;
  for (uint32_t g = 0; g < n_seg; ++g)
    if (offsets[g + 1] < offsets[g]) return ORC_E_INVAL;
  for (uint64_t p = 0; p < n_keys; ++p)
    if (keys[p] == SENTINEL) return ORC_E_BADKEY;

  // union of the referenced keys, ascending, and occurrence -> unique index
  std::vector<uint64_t> uniq(keys, keys + n_keys);
  std::sort(uniq.begin(), uniq.end());
  uniq.erase(std::unique(uniq.begin(), uniq.end()), uniq.end());
  std::vector<uint32_t> inverse(n_keys);
  for (uint64_t p = 0; p < n_keys; ++p)
    inverse[p] = (uint32_t)(std::lower_bound(uniq.begin(), uniq.end(), keys[p]) - uniq.begin());

  // insert-on-miss, rows in order of first occurrence
  std::vector<uint64_t> fresh;
  {
    std::unordered_set<uint64_t> seen;
    for (uint64_t p = 0; p < n_keys; ++p) {
      if (t->row_of.find(keys[p]) != t->row_of.end()) continue;
      if (seen.insert(keys[p]).second) fresh.push_back(keys[p]);
    }
  }
  if (t->n_rows + fresh.size() > t->R) return ORC_E_FULL;
  const float scale = init_scale(t->init_std);
  for (uint64_t key : fresh) {
    uint32_t r = (uint32_t)t->n_rows++;
    t->row_of[key] = r;
    t->key_of_row.push_back(key);
    for (uint32_t j = 0; j < t->W; ++j) {
      for (uint32_t d = 0; d < D; ++d) {
        t->x[j].push_back(init_value(t->seed, key, d, scale));
        t->m[j].push_back(0.0f);
        t->v[j].push_back(t->variant == VAR_KINGMA ? 0.0f : t->eps);
      }
      t->pending[j].push_back(0);
    }
    if (t->kstep && t->variant != VAR_PROSE)
      for (uint32_t d = 0; d < D; ++d) t->vhat.push_back(t->eps);
    t->touched.push_back(0);
  }
  t->n_new_last = fresh.size();

  std::vector<uint32_t> rows(uniq.size());
  for (size_t u = 0; u < uniq.size(); ++u) rows[u] = t->row_of[uniq[u]];

  // pooling: sum in binary64 in CSR order, rounded once
  const std::vector<float>& x = t->x[replica];
  std::vector<double> acc(D);
  for (uint32_t g = 0; g < n_seg; ++g) {
    std::fill(acc.begin(), acc.end(), 0.0);
    for (uint32_t p = offsets[g]; p < offsets[g + 1]; ++p) {
      const float* row = &x[(size_t)rows[inverse[p]] * D];
      for (uint32_t d = 0; d < D; ++d) acc[d] += (double)row[d];
    }
    for (uint32_t d = 0; d < D; ++d) pooled[(size_t)g * D + d] = (float)acc[d];
  }

  t->uniq.swap(uniq);
  t->rows.swap(rows);
  t->inverse.swap(inverse);
  t->offsets.assign(offsets, offsets + n_seg + 1);
  t->batch_valid = true;
  t->batch_replica = replica;
  return ORC_OK;
}

// Push: per-key gradient sums, then one Adam step per distinct key.
int orc_push_adam(void* h, uint32_t replica, const float* grad_pooled, uint32_t mode) {
  Table* t = (Table*)h;
  const uint32_t D = t->D;
  if (replica >= t->W) return ORC_E_INVAL;
  if (mode != STEP_LOCAL && mode != STEP_MERGE_PENDING) return ORC_E_INVAL;
  if ((!t->kstep || t->variant == VAR_PROSE) && mode != STEP_LOCAL) return ORC_E_INVAL;
  if (!t->batch_valid || t->batch_replica != replica) return ORC_E_STATE;
  t->batch_valid = false;
  ++t->n_push;

  const size_t U = t->uniq.size();
  const uint32_t n_seg = (uint32_t)t->offsets.size() - 1;
  std::vector<double> gsum(U * D, 0.0);
  for (uint32_t g = 0; g < n_seg; ++g)
    for (uint32_t p = t->offsets[g]; p < t->offsets[g + 1]; ++p) {
      double* dst = &gsum[(size_t)t->inverse[p] * D];
      const float* src = &grad_pooled[(size_t)g * D];
      for (uint32_t d = 0; d < D; ++d) dst[d] += (double)src[d];
    }

  const double b1 = (double)t->b1, b2 = (double)t->b2, lr = (double)t->lr;
  std::vector<float>&x = t->x[replica], &m = t->m[replica], &v = t->v[replica];
  for (size_t u = 0; u < U; ++u) {
    const size_t r = t->rows[u];
    for (uint32_t d = 0; d < D; ++d) {
      const size_t i = r * D + d;
      const double g = gsum[u * D + d];
      if (t->variant == VAR_ADAGRAD) {  // v holds the accumulator G
        v[i] = (float)((double)v[i] + g * g);
        x[i] = (float)((double)x[i] - lr * g / std::sqrt((double)v[i]));
        continue;
      }
      m[i] = (float)(b1 * (double)m[i] + (1.0 - b1) * g);
      v[i] = (float)(b2 * (double)v[i] + (1.0 - b2) * (g * g));
      if (t->variant == VAR_KINGMA) {
        const double mhat = (double)m[i] / (1.0 - std::pow(b1, (double)t->n_push));
        const double vhat = (double)v[i] / (1.0 - std::pow(b2, (double)t->n_push));
        x[i] = (float)((double)x[i] - lr * mhat / (std::sqrt(vhat) + (double)t->eps));
      } else if (!t->kstep || t->variant == VAR_PROSE) {
        x[i] = (float)((double)x[i] - lr * (double)m[i] / std::sqrt((double)v[i]));
      } else if (mode == STEP_LOCAL) {
        x[i] = (float)((double)x[i] - lr * (double)m[i] / std::sqrt((double)t->vhat[i]));
      }
    }
    if (t->kstep) {
      t->touched[r] = 1;
      if (mode == STEP_MERGE_PENDING) t->pending[replica][r] = 1;
    }
  }
  return ORC_OK;
}

// k-step merge over the rows touched since the previous merge.
int orc_kstep_merge(void* h) {
  Table* t = (Table*)h;
  if (!t->kstep) return ORC_E_INVAL;
  const uint32_t D = t->D, W = t->W;
  const double lr = (double)t->lr;
  for (size_t r = 0; r < t->n_rows; ++r) {
    if (!t->touched[r]) continue;
    for (uint32_t d = 0; d < D; ++d) {
      const size_t i = r * D + d;
      double vs = 0.0;
      for (uint32_t j = 0; j < W; ++j) vs += (double)t->v[j][i];
      const float vbar = (float)(vs / (double)W);
      if (t->variant == VAR_PROSE) {
        double xs = 0.0;
        for (uint32_t j = 0; j < W; ++j) xs += (double)t->x[j][i];
        const float xbar = (float)(xs / (double)W);
        for (uint32_t j = 0; j < W; ++j) {
          t->x[j][i] = xbar;
          t->v[j][i] = vbar;
        }
        continue;
      }
      t->vhat[i] = vbar;
      const double den = std::sqrt((double)t->vhat[i]);
      double xs = 0.0;
      for (uint32_t j = 0; j < W; ++j) {
        double y = (double)t->x[j][i];
        if (t->pending[j][r]) y -= lr * (double)t->m[j][i] / den;
        xs += y;
      }
      const float xbar = (float)(xs / (double)W);
      for (uint32_t j = 0; j < W; ++j) t->x[j][i] = xbar;
    }
    for (uint32_t j = 0; j < W; ++j) t->pending[j][r] = 0;
    t->touched[r] = 0;
  }
  return ORC_OK;
}

// Lookup-only pooling (prediction with a trained table: the embedding layer of Section 2.1 without the
// insert-on-miss of training): keys that are not in the table contribute nothing; the table, its
// pending batch and every counter stay as they are.
int orc_lookup_pool(void* h, uint32_t replica, const uint64_t* keys, uint64_t n_keys, const uint32_t* offsets,
                    uint32_t n_seg, float* pooled) {
  Table* t = (Table*)h;
  const uint32_t D = t->D;
  if (replica >= t->W) return ORC_E_INVAL;
  if (offsets[0] != 0 || offsets[n_seg] != n_keys) return ORC_E_INVAL;
  for (uint32_t g = 0; g < n_seg; ++g)
    if (offsets[g + 1] < offsets[g]) return ORC_E_INVAL;
  for (uint64_t p = 0; p < n_keys; ++p)
    if (keys[p] == SENTINEL) return ORC_E_BADKEY;
  const std::vector<float>& x = t->x[replica];
  std::vector<double> acc(D);
  for (uint32_t g = 0; g < n_seg; ++g) {
    std::fill(acc.begin(), acc.end(), 0.0);
    for (uint32_t p = offsets[g]; p < offsets[g + 1]; ++p) {
      auto it = t->row_of.find(keys[p]);
      if (it == t->row_of.end()) continue;
      const float* row = &x[(size_t)it->second * D];
      for (uint32_t d = 0; d < D; ++d) acc[d] += (double)row[d];
    }
    for (uint32_t d = 0; d < D; ++d) pooled[(size_t)g * D + d] = (float)acc[d];
  }
  return ORC_OK;
}

// Empties the table (Algorithm 1: the hash table holds one batch's working parameters; the next batch
// brings its own): no rows, no keys, nothing pending; hyper-parameters and the step count stay.
int orc_table_clear(void* h) {
  Table* t = (Table*)h;
  t->n_rows = 0;
  t->row_of.clear();
  t->key_of_row.clear();
  for (uint32_t j = 0; j < t->W; ++j) {
    t->x[j].clear();
    t->m[j].clear();
    t->v[j].clear();
    t->pending[j].clear();
  }
  t->vhat.clear();
  t->touched.clear();
  t->batch_valid = false;
  t->n_new_last = 0;
  return ORC_OK;
}

// Working-set load (Algorithm 1: insert_into_hash_table of a parameter partition): keys not in the
// table get new rows in the order given, keys already there are overwritten; every replica gets
// the same state and the shared denominator of the row is set to v.
int orc_table_load(void* h, const uint64_t* keys, uint64_t n, const float* x, const float* m, const float* v) {
  Table* t = (Table*)h;
  const uint32_t D = t->D;
  for (uint64_t p = 0; p < n; ++p)
    if (keys[p] == SENTINEL) return ORC_E_BADKEY;
  {
    std::unordered_set<uint64_t> fresh;
    for (uint64_t p = 0; p < n; ++p)
      if (t->row_of.find(keys[p]) == t->row_of.end()) fresh.insert(keys[p]);
    if (t->n_rows + fresh.size() > t->R) return ORC_E_FULL;
  }
  t->batch_valid = false;
  const bool has_vhat = t->kstep && t->variant != VAR_PROSE;
  for (uint64_t p = 0; p < n; ++p) {
    auto it = t->row_of.find(keys[p]);
    uint32_t r;
    if (it == t->row_of.end()) {
      r = (uint32_t)t->n_rows++;
      t->row_of[keys[p]] = r;
      t->key_of_row.push_back(keys[p]);
      for (uint32_t j = 0; j < t->W; ++j) {
        t->x[j].resize((size_t)t->n_rows * D);
        t->m[j].resize((size_t)t->n_rows * D);
        t->v[j].resize((size_t)t->n_rows * D);
        t->pending[j].push_back(0);
      }
      if (has_vhat) t->vhat.resize((size_t)t->n_rows * D);
      t->touched.push_back(0);
    } else {
      r = it->second;
    }
    for (uint32_t j = 0; j < t->W; ++j)
      for (uint32_t d = 0; d < D; ++d) {
        t->x[j][(size_t)r * D + d] = x[p * D + d];
        t->m[j][(size_t)r * D + d] = (t->variant == VAR_ADAGRAD) ? 0.0f : m[p * D + d];
        t->v[j][(size_t)r * D + d] = v[p * D + d];
      }
    if (has_vhat)
      for (uint32_t d = 0; d < D; ++d) t->vhat[(size_t)r * D + d] = v[p * D + d];
  }
  return ORC_OK;
}

// Collection of rows by key, without inserting (Algorithm 1: pull_updates_peer_GPU).
int orc_table_collect(void* h, uint32_t replica, const uint64_t* keys, uint64_t n, float* x, float* m, float* v,
                      uint32_t* found) {
  Table* t = (Table*)h;
  if (replica >= t->W) return ORC_E_INVAL;
  const uint32_t D = t->D;
  for (uint64_t p = 0; p < n; ++p) {
    auto it = t->row_of.find(keys[p]);
    const bool hit = it != t->row_of.end();
    if (found) found[p] = hit ? 1u : 0u;
    for (uint32_t d = 0; d < D; ++d) {
      const size_t i = hit ? (size_t)it->second * D + d : 0;
      if (x) x[p * D + d] = hit ? t->x[replica][i] : 0.0f;
      if (m) m[p * D + d] = hit ? t->m[replica][i] : 0.0f;
      if (v) v[p * D + d] = hit ? t->v[replica][i] : 0.0f;
    }
  }
  return ORC_OK;
}

// Dedup result of the last pull: ascending distinct keys, their rows, and the
// index of every occurrence's key in that list.
int orc_batch_export(void* h, uint64_t* uniq, uint32_t* rows, uint32_t* inverse) {
  Table* t = (Table*)h;
  if (!t->batch_valid) return ORC_E_STATE;
  if (uniq) std::memcpy(uniq, t->uniq.data(), t->uniq.size() * sizeof(uint64_t));
  if (rows) std::memcpy(rows, t->rows.data(), t->rows.size() * sizeof(uint32_t));
  if (inverse) std::memcpy(inverse, t->inverse.data(), t->inverse.size() * sizeof(uint32_t));
  return ORC_OK;
}

// Table contents in row order: keys[n_rows], x/m/v[n_rows*D] of one replica, shared v.
int orc_table_export(void* h, uint32_t replica, uint64_t* keys, float* x, float* m, float* v,
                     float* vhat) {
  Table* t = (Table*)h;
  if (replica >= t->W) return ORC_E_INVAL;
  const size_t n = (size_t)t->n_rows * t->D;
  if (keys) std::memcpy(keys, t->key_of_row.data(), t->n_rows * sizeof(uint64_t));
  if (x) std::memcpy(x, t->x[replica].data(), n * sizeof(float));
  if (m) std::memcpy(m, t->m[replica].data(), n * sizeof(float));
  if (v) std::memcpy(v, t->v[replica].data(), n * sizeof(float));
  if (vhat) {
    if (!t->kstep || t->variant == VAR_PROSE) return ORC_E_INVAL;
    std::memcpy(vhat, t->vhat.data(), n * sizeof(float));
  }
  return ORC_OK;
}

}  // extern "C"
