// Reference ("oracle") implementation of the HBM-PS mini-batch pull/push.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plainly
// written definition of what the GPU library must compute.  Only the test
// suite, the smoke check and the benchmark's CPU-baseline leg may use it; the
// product library never links, loads or calls it, and the two share no code.
//
// What it follows (paper: "Distributed Hierarchical GPU Parameter Server for
// Massive Scale Deep Learning Ads Systems", MLSys 2020):
//   * Section 4.1, "Local GPU hash table": a keyed table whose capacity is
//     fixed when it is built, with operations insert / get / accumulate.
//   * Algorithm 1: insert the working parameters, then per mini-batch pull the
//     referenced parameters, train, push the updates back; finally collect the
//     table's content (dump).
//   * Section 3, "Workflow": the union of referenced parameters of a batch
//     (here: sorted unique keys plus, per occurrence, the rank of its key).
//   * Section 4.1, "Operations": accumulate adds the pushed values onto the
//     parameters their keys reference.  Here the pushed values are upstream
//     gradients of sum-pooled bags; they are summed per unique key and one
//     Adagrad step is taken per touched row (the optimizer is this build's
//     reading; the paper leaves the update rule to the trainer).
//
// Arithmetic: every sum and the optimizer step are evaluated in double from
// the stored float32 values and rounded to float32 once, when stored.
// The row initialiser is defined in float32 (two separately rounded
// operations), so it has exactly one correct bit pattern.
// Row format bfloat16 (an extension, not from the paper: its rows are float32): a weight
// is additionally rounded to the nearest bfloat16 value (ties to even) whenever it is
// stored, and read back as that value; accumulators stay float32.
//
// Build: g++ -O2 -ffp-contract=off -shared -fPIC (see oracle/__init__.py).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

namespace {

constexpr uint64_t kReservedKey = ~uint64_t(0);

enum Status { OK = 0, EINVAL = -1, EFULL = -2, ERESERVED = -3, ESTATE = -4 };
enum OptKind { ADAGRAD_ROWWISE = 0, ADAGRAD_ELEMENTWISE = 1 };
enum RowFormat { ROWS_F32 = 0, ROWS_BF16 = 1 };

// The nearest bfloat16 value (1 sign, 8 exponent, 7 fraction bits: the upper half of a
// float32), ties to even, as a float32.
float nearest_bf16(float x) {
  if (std::isnan(x)) return x;
  uint32_t u;
  std::memcpy(&u, &x, 4);
  const uint32_t dropped = u & 0xFFFFu;
  uint32_t kept = u >> 16;
  if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u))) kept += 1;   // carries into the exponent correctly
  u = kept << 16;
  std::memcpy(&x, &u, 4);
  return x;
}

// SplitMix64 output function (Steele, Lea, Flood: "Fast splittable
// pseudorandom number generators", 2014) for the state x.
uint64_t mix(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

struct Table {
  uint64_t capacity;
  uint32_t dim;
  int opt;
  float lr, eps, init_acc, init_range;
  uint64_t init_seed;
  uint32_t acc_len;                       // 1 (row-wise) or dim (element-wise)
  int row_format = ROWS_F32;
  // what a weight becomes when it is stored
  float stored(float x) const { return row_format == ROWS_BF16 ? nearest_bf16(x) : x; }
  std::unordered_map<uint64_t, uint64_t> index;   // key -> row number
  std::vector<uint64_t> row_key;
  std::vector<float> w;                   // [rows, dim]
  std::vector<float> acc;                 // [rows, acc_len]
  std::vector<uint8_t> dirty;             // [rows]: updated since the last dirty dump
  uint64_t implicit_rows = 0;             // declared-resident rows not materialised
  uint64_t implicit_seen = 0;             // ... of which materialised since

  // context of the outstanding pull
  bool pulled = false;
  std::vector<uint64_t> uniq;
  std::vector<int32_t> inverse;
  std::vector<int32_t> bag_of;
  std::vector<int32_t> bag_len;           // occurrences in each bag of the outstanding pull
  uint64_t n_bags = 0;
  int mean_pooling = 0;                   // 0: a bag's rows are summed; 1: averaged

  uint64_t size() const { return row_key.size() + implicit_rows - implicit_seen; }
};

// Deterministic initial weights of a new row: element j of key's row is
// uniform on [-init_range, init_range) with 24 random bits, as two float32
// operations that are each rounded (no fused multiply-add).
void init_weights(const Table& t, uint64_t key, float* out) {
  const uint64_t base = mix(key ^ t.init_seed);
  const float two_a = t.init_range * 2.0f;
  for (uint32_t j = 0; j < t.dim; ++j) {
    const uint64_t r = mix(base + j);
    const float u = (float)(uint32_t)(r >> 40) * 0x1.0p-24f;   // [0, 1), exact
    volatile float scaled = u * two_a;                          // rounded product
    out[j] = scaled - t.init_range;                             // rounded difference
  }
}

uint64_t add_row(Table& t, uint64_t key) {
  const uint64_t r = t.row_key.size();
  t.index.emplace(key, r);
  t.row_key.push_back(key);
  t.w.resize((r + 1) * t.dim);
  init_weights(t, key, &t.w[r * t.dim]);
  for (uint32_t j = 0; j < t.dim; ++j) t.w[r * t.dim + j] = t.stored(t.w[r * t.dim + j]);
  t.acc.resize((r + 1) * t.acc_len, t.init_acc);
  t.dirty.resize(r + 1, 0);
  return r;
}

// Sorted unique keys and, per occurrence, the rank of its key among them.
void dedup(const uint64_t* keys, uint64_t n, std::vector<uint64_t>& uniq,
           std::vector<int32_t>& inverse) {
  uniq.assign(keys, keys + n);
  std::sort(uniq.begin(), uniq.end());
  uniq.erase(std::unique(uniq.begin(), uniq.end()), uniq.end());
  inverse.resize(n);
  for (uint64_t i = 0; i < n; ++i)
    inverse[i] = (int32_t)(std::lower_bound(uniq.begin(), uniq.end(), keys[i]) - uniq.begin());
}

}  // namespace

extern "C" {

uint64_t hpo_mix(uint64_t x) { return mix(x); }

void* hpo_create(uint64_t capacity, uint32_t dim, int opt, float lr, float eps, float init_acc,
                 float init_range, uint64_t init_seed) {
  if (capacity == 0 || dim == 0 || (opt != ADAGRAD_ROWWISE && opt != ADAGRAD_ELEMENTWISE))
    return nullptr;
  Table* t = new Table();
  t->capacity = capacity;
  t->dim = dim;
  t->opt = opt;
  t->lr = lr;
  t->eps = eps;
  t->init_acc = init_acc;
  t->init_range = init_range;
  t->init_seed = init_seed;
  t->acc_len = (opt == ADAGRAD_ELEMENTWISE) ? dim : 1;
  return t;
}

void hpo_destroy(void* h) { delete static_cast<Table*>(h); }

// Algorithm 1 builds the HBM table anew for every batch of the outer loop (insert the
// batch's working parameters, run its mini-batches, hand the updates to the host tier):
// this empties the table for the next batch.  Settings (optimizer, pooling, row format)
// stay.
int hpo_clear(void* h) {
  Table& t = *static_cast<Table*>(h);
  if (t.pulled) return ESTATE;
  t.index.clear();
  t.row_key.clear();
  t.w.clear();
  t.acc.clear();
  t.dirty.clear();
  t.implicit_rows = t.implicit_seen = 0;
  return OK;
}

// How weights are stored: float32 (0, the default) or bfloat16 (1).  Only while the table
// is empty.
int hpo_set_row_format(void* h, int format) {
  Table& t = *static_cast<Table*>(h);
  if (format != ROWS_F32 && format != ROWS_BF16) return EINVAL;
  if (t.size() != 0) return ESTATE;
  t.row_format = format;
  return OK;
}

float hpo_nearest_bf16(float x) { return nearest_bf16(x); }

uint64_t hpo_size(void* h) { return static_cast<Table*>(h)->size(); }
uint32_t hpo_acc_len(void* h) { return static_cast<Table*>(h)->acc_len; }

// The row a new key gets, as the table stores it.
void hpo_init_row(void* h, uint64_t key, float* out) {
  const Table& t = *static_cast<Table*>(h);
  init_weights(t, key, out);
  for (uint32_t j = 0; j < t.dim; ++j) out[j] = t.stored(out[j]);
}

// Declares that n further keys are resident with untouched (initial) rows
// without storing them.  Untouched rows are a pure function of the key, so a
// test that knows which keys those are materialises them on first use with
// hpo_materialize; the size accounting is as if all had been inserted.
int hpo_declare_resident(void* h, uint64_t n) {
  Table& t = *static_cast<Table*>(h);
  if (t.size() + n > t.capacity) return EFULL;
  t.implicit_rows += n;
  return OK;
}

// Turns declared-resident keys into stored rows (initial contents).
int hpo_materialize(void* h, const uint64_t* keys, uint64_t n) {
  Table& t = *static_cast<Table*>(h);
  for (uint64_t i = 0; i < n; ++i) {
    if (keys[i] == kReservedKey) return ERESERVED;
    if (t.index.count(keys[i])) continue;
    if (t.implicit_seen >= t.implicit_rows) return ESTATE;
    add_row(t, keys[i]);
    t.implicit_seen += 1;
  }
  return OK;
}

// Section 4.1 "insert" / Algorithm 1 "insert_into_hashtable": bulk load.
// weights == NULL: a key that is absent gets its initial row, a present key is
// left as it is.  weights != NULL: the row is created or overwritten with the
// given weights (and accumulators, when acc != NULL; else the initial value).
int hpo_insert(void* h, const uint64_t* keys, uint64_t n, const float* weights, const float* acc) {
  Table& t = *static_cast<Table*>(h);
  for (uint64_t i = 0; i < n; ++i)
    if (keys[i] == kReservedKey) return ERESERVED;
  for (uint64_t i = 0; i < n; ++i) {
    auto it = t.index.find(keys[i]);
    uint64_t r;
    if (it == t.index.end()) {
      if (t.size() >= t.capacity) return EFULL;
      r = add_row(t, keys[i]);
    } else {
      r = it->second;
      if (!weights) continue;
    }
    if (weights) {
      for (uint32_t j = 0; j < t.dim; ++j) t.w[r * t.dim + j] = t.stored(weights[i * t.dim + j]);
      for (uint32_t j = 0; j < t.acc_len; ++j)
        t.acc[r * t.acc_len + j] = acc ? acc[i * t.acc_len + j] : t.init_acc;
    }
  }
  return OK;
}

// Section 3: the union of the parameters a batch references.
int hpo_dedup(const uint64_t* keys, uint64_t n, uint64_t* uniq_out, int32_t* inverse_out,
              uint64_t* n_uniq) {
  std::vector<uint64_t> u;
  std::vector<int32_t> inv;
  dedup(keys, n, u, inv);
  std::copy(u.begin(), u.end(), uniq_out);
  std::copy(inv.begin(), inv.end(), inverse_out);
  *n_uniq = u.size();
  return OK;
}

// Algorithm 1 "pull_HBM-PS_kernel": look up (or create) the row of every
// referenced key, then sum the rows of each bag (example x slot).
//   offsets[n_bags + 1]: bag b owns occurrences offsets[b] .. offsets[b+1]-1.
//   pooled[n_bags, dim]; an empty bag gives zeros.
// A key that occurs twice in a bag is added twice.
int hpo_pull(void* h, const uint64_t* keys, uint64_t n, const int32_t* offsets, uint64_t n_bags,
             float* pooled, uint64_t* n_uniq, uint64_t* n_inserted) {
  Table& t = *static_cast<Table*>(h);
  if (offsets[0] != 0 || (uint64_t)offsets[n_bags] != n) return EINVAL;
  for (uint64_t b = 0; b < n_bags; ++b)
    if (offsets[b + 1] < offsets[b]) return EINVAL;
  for (uint64_t i = 0; i < n; ++i)
    if (keys[i] == kReservedKey) return ERESERVED;

  dedup(keys, n, t.uniq, t.inverse);
  uint64_t inserted = 0;
  std::vector<uint64_t> row_of(t.uniq.size());
  int status = OK;
  for (size_t u = 0; u < t.uniq.size(); ++u) {
    auto it = t.index.find(t.uniq[u]);
    if (it != t.index.end()) {
      row_of[u] = it->second;
    } else if (t.size() >= t.capacity) {
      status = EFULL;
      break;
    } else {
      row_of[u] = add_row(t, t.uniq[u]);
      ++inserted;
    }
  }
  *n_uniq = t.uniq.size();
  *n_inserted = inserted;
  if (status != OK) { t.pulled = false; return status; }

  t.bag_of.resize(n);
  t.bag_len.assign(n_bags, 0);
  std::vector<double> sum(t.dim);
  for (uint64_t b = 0; b < n_bags; ++b) {
    std::fill(sum.begin(), sum.end(), 0.0);
    for (int32_t i = offsets[b]; i < offsets[b + 1]; ++i) {
      t.bag_of[i] = (int32_t)b;
      const float* row = &t.w[row_of[t.inverse[i]] * t.dim];
      for (uint32_t j = 0; j < t.dim; ++j) sum[j] += (double)row[j];
    }
    const int32_t len = offsets[b + 1] - offsets[b];
    t.bag_len[b] = len;
    const double scale = t.mean_pooling && len > 0 ? 1.0 / (double)len : 1.0;
    for (uint32_t j = 0; j < t.dim; ++j) pooled[b * t.dim + j] = (float)(sum[j] * scale);
  }
  t.n_bags = n_bags;
  t.pulled = true;
  return OK;
}

// Pooling of the bags: sum (0, the default) or mean (1: the pooled row is the average of
// the bag's rows, and the bag's upstream gradient reaches each of its occurrences divided
// by the bag's length).  Not from the paper, which leaves the embedding layer's reduction
// to the trainer; takes effect from the next pull on.
int hpo_set_pooling(void* h, int mean) {
  Table& t = *static_cast<Table*>(h);
  if (t.pulled) return ESTATE;
  if (mean != 0 && mean != 1) return EINVAL;
  t.mean_pooling = mean;
  return OK;
}

// Context of the last pull, for checking dedup results.
int hpo_last_unique(void* h, uint64_t* uniq_out, int32_t* inverse_out) {
  Table& t = *static_cast<Table*>(h);
  if (!t.pulled) return ESTATE;
  if (uniq_out) std::copy(t.uniq.begin(), t.uniq.end(), uniq_out);
  if (inverse_out) std::copy(t.inverse.begin(), t.inverse.end(), inverse_out);
  return OK;
}

// Algorithm 1 "push_parameters_updates_back_kernel" / Algorithm 2's local
// accumulate: the gradient of a sum-pooled bag reaches each of its key
// occurrences unchanged, so the gradient of a row is the sum of the bag
// gradients over all occurrences of its key.  Each touched row then takes ONE
// Adagrad step:
//   row-wise:      G' = G + (1/dim) * sum_j g_j^2 ;  w_j' = w_j - lr * g_j / (sqrt(G') + eps)
//   element-wise:  G_j' = G_j + g_j^2             ;  w_j' = w_j - lr * g_j / (sqrt(G_j') + eps)
int hpo_push(void* h, const float* grads) {
  Table& t = *static_cast<Table*>(h);
  if (!t.pulled) return ESTATE;
  const size_t U = t.uniq.size(), n = t.inverse.size();
  // occurrences of each unique key, in ascending occurrence order
  std::vector<uint64_t> start(U + 1, 0);
  for (size_t i = 0; i < n; ++i) start[t.inverse[i] + 1] += 1;
  for (size_t u = 0; u < U; ++u) start[u + 1] += start[u];
  std::vector<uint64_t> fill(start.begin(), start.end() - 1), occ(n);
  for (size_t i = 0; i < n; ++i) occ[fill[t.inverse[i]]++] = i;

  std::vector<double> g(t.dim);
  const double lr = (double)t.lr, eps = (double)t.eps;
  for (size_t u = 0; u < U; ++u) {
    std::fill(g.begin(), g.end(), 0.0);
    for (uint64_t p = start[u]; p < start[u + 1]; ++p) {
      const int32_t bag = t.bag_of[occ[p]];
      const float* row = grads + (uint64_t)bag * t.dim;
      // mean pooling: an occurrence's share of its bag's gradient is 1 / (bag length)
      const double share = t.mean_pooling ? 1.0 / (double)t.bag_len[bag] : 1.0;
      for (uint32_t j = 0; j < t.dim; ++j) g[j] += (double)row[j] * share;
    }
    const uint64_t r = t.index.at(t.uniq[u]);
    float* w = &t.w[r * t.dim];
    float* a = &t.acc[r * t.acc_len];
    if (t.opt == ADAGRAD_ROWWISE) {
      double ss = 0.0;
      for (uint32_t j = 0; j < t.dim; ++j) ss += g[j] * g[j];
      const double G = (double)a[0] + ss / (double)t.dim;
      const double denom = std::sqrt(G) + eps;
      for (uint32_t j = 0; j < t.dim; ++j) w[j] = t.stored((float)((double)w[j] - lr * g[j] / denom));
      a[0] = (float)G;
    } else {
      for (uint32_t j = 0; j < t.dim; ++j) {
        const double G = (double)a[j] + g[j] * g[j];
        w[j] = t.stored((float)((double)w[j] - lr * g[j] / (std::sqrt(G) + eps)));
        a[j] = (float)G;
      }
    }
    t.dirty[r] = 1;
  }
  t.pulled = false;
  return OK;
}

// Section 4.1 "Operations", accumulate, in the paper's literal form: the input is a
// collection of (key, value row) pairs and every value row is added onto the
// parameter row its key references; a key that comes several times receives the
// sum of its rows.  Keys the table does not hold are skipped and counted
// (*n_absent): nothing is created (Algorithm 1 inserts the working set before
// the mini-batch loop, so a training run never meets one).  The optimizer state
// is not touched.
int hpo_accumulate(void* h, const uint64_t* keys, uint64_t n, const float* values,
                   uint64_t* n_absent) {
  Table& t = *static_cast<Table*>(h);
  if (t.pulled) return ESTATE;
  for (uint64_t i = 0; i < n; ++i)
    if (keys[i] == kReservedKey) return ERESERVED;
  std::vector<uint64_t> uniq;
  std::vector<int32_t> inverse;
  dedup(keys, n, uniq, inverse);
  std::vector<double> sum(uniq.size() * (size_t)t.dim, 0.0);
  for (uint64_t i = 0; i < n; ++i)
    for (uint32_t j = 0; j < t.dim; ++j)
      sum[(size_t)inverse[i] * t.dim + j] += (double)values[i * t.dim + j];
  uint64_t absent = 0;
  for (size_t u = 0; u < uniq.size(); ++u) {
    auto it = t.index.find(uniq[u]);
    if (it == t.index.end()) { ++absent; continue; }
    float* w = &t.w[it->second * t.dim];
    for (uint32_t j = 0; j < t.dim; ++j) w[j] = t.stored((float)((double)w[j] + sum[u * t.dim + j]));
    t.dirty[it->second] = 1;
  }
  if (n_absent) *n_absent = absent;
  return OK;
}

// Section 4.1 "get": read rows by key, no insertion.
int hpo_get(void* h, const uint64_t* keys, uint64_t n, float* w_out, float* acc_out,
            uint8_t* found_out) {
  Table& t = *static_cast<Table*>(h);
  for (uint64_t i = 0; i < n; ++i) {
    auto it = t.index.find(keys[i]);
    found_out[i] = it != t.index.end();
    if (!found_out[i]) continue;
    std::memcpy(w_out + i * t.dim, &t.w[it->second * t.dim], sizeof(float) * t.dim);
    std::memcpy(acc_out + i * t.acc_len, &t.acc[it->second * t.acc_len], sizeof(float) * t.acc_len);
  }
  return OK;
}

uint64_t hpo_stored_rows(void* h) { return static_cast<Table*>(h)->row_key.size(); }

// Algorithm 1 "pull_updates_HBM-PS": every stored row, ascending by key.
int hpo_dump(void* h, uint64_t* keys_out, float* w_out, float* acc_out, uint64_t max_rows,
             uint64_t* n_rows) {
  Table& t = *static_cast<Table*>(h);
  const uint64_t R = t.row_key.size();
  *n_rows = R;
  if (R > max_rows) return EINVAL;
  std::vector<uint64_t> order(R);
  for (uint64_t r = 0; r < R; ++r) order[r] = r;
  std::sort(order.begin(), order.end(),
            [&](uint64_t a, uint64_t b) { return t.row_key[a] < t.row_key[b]; });
  for (uint64_t o = 0; o < R; ++o) {
    const uint64_t r = order[o];
    keys_out[o] = t.row_key[r];
    std::memcpy(w_out + o * t.dim, &t.w[r * t.dim], sizeof(float) * t.dim);
    std::memcpy(acc_out + o * t.acc_len, &t.acc[r * t.acc_len], sizeof(float) * t.acc_len);
  }
  return OK;
}

// Section 4 (MEM-PS side of Algorithm 1's last step): the host tier collects the
// UPDATES of the HBM tier.  This variant hands over only the rows that a push or
// an accumulate has changed since the previous call (or since the table was
// built), ascending by key, and forgets the marks of the rows it handed over.
// Rows that were only inserted or only created by a pull are not updates.
int hpo_dump_dirty(void* h, uint64_t* keys_out, float* w_out, float* acc_out, uint64_t max_rows,
                   uint64_t* n_rows) {
  Table& t = *static_cast<Table*>(h);
  std::vector<uint64_t> order;
  for (uint64_t r = 0; r < t.row_key.size(); ++r)
    if (t.dirty[r]) order.push_back(r);
  *n_rows = order.size();
  if (order.size() > max_rows) return EINVAL;
  std::sort(order.begin(), order.end(),
            [&](uint64_t a, uint64_t b) { return t.row_key[a] < t.row_key[b]; });
  for (uint64_t o = 0; o < order.size(); ++o) {
    const uint64_t r = order[o];
    keys_out[o] = t.row_key[r];
    std::memcpy(w_out + o * t.dim, &t.w[r * t.dim], sizeof(float) * t.dim);
    std::memcpy(acc_out + o * t.acc_len, &t.acc[r * t.acc_len], sizeof(float) * t.acc_len);
    t.dirty[r] = 0;
  }
  return OK;
}

}  // extern "C"
