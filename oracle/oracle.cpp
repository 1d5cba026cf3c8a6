// CPU checker for the sparse-embedding path (TEST INFRASTRUCTURE, not a product path).
//
// A plain, single-threaded, obviously-correct statement of what one device
// computes for the embedding layer of a generative recommendation model:
// tagged IDs of merged tables (Sec. 3.2, Eq. 8), ID deduplication with inverse
// indices (Sec. 3.3), a dynamic key -> embedding-row table with real-time
// insertion and deletion (Sec. 3.1), per-ID gradient aggregation and an update
// of the activated rows only (Sec. 2 "Backward Update"; App. C "Gradient
// Accumulation").  The table is a std::unordered_map, the unique is a
// std::sort; there is no blocking, fusion or reordering.
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call
// this library.  It shares no source, header, table or constant generator with
// the GPU library.
//
// Parity pins live in tests/test_oracle_*.py.  Parts whose definition the paper
// leaves open (row initialisation, the optimizer, the eviction predicate, pooling,
// hot rows) follow the reading stated at each function; no function here is
// "parity unpinned".
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

namespace {

constexpr int kF32 = 0;
constexpr int kBF16 = 1;

struct Row {
    std::vector<float> w;   // bf16 tables keep bf16-representable floats
    float acc = 0.0f;       // row-wise Adagrad accumulator
    uint32_t last_seen = 0; // step of the last find-or-insert that touched the key
    uint32_t freq = 0;      // number of find-or-insert elements that touched the key
    std::vector<float> m, v; // Adam moments (empty = all zero)
    bool hot = false;        // 16-bit table only: w holds an fp32 master instead of 16-bit values
};

struct Table {
    int dim;
    int dtype;
    float init_scale;
    std::unordered_map<uint64_t, Row> map;
    int64_t hot_capacity = 0; // masters the hot store can hold (0 = no hot store)
    int64_t hot_used = 0;
};

// ---- bf16 <-> float, written out (round to nearest, ties to even) ---------
inline float bf16_bits_to_float(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}
inline uint16_t float_to_bf16_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    uint32_t keep_lsb = (u >> 16) & 1u;
    u += 0x7FFFu + keep_lsb;
    return static_cast<uint16_t>(u >> 16);
}
// One rounding from double straight to a bf16-representable float (normal range).
inline float double_to_bf16_float(double d) {
    uint64_t u;
    std::memcpy(&u, &d, 8);
    const int drop = 52 - 7;
    uint64_t keep_lsb = (u >> drop) & 1ull;
    u += ((1ull << (drop - 1)) - 1ull) + keep_lsb;
    u &= ~((1ull << drop) - 1ull);
    double r;
    std::memcpy(&r, &u, 8);
    return static_cast<float>(r); // exact: r has 8 significant bits
}

// ---- key-seeded row initialisation ----------------------------------------
// Element j of the row of `key` is the (j+1)-th output of a splitmix64 stream
// seeded with the tagged key, mapped to a 24-bit signed integer and scaled by
// init_scale * 2^-23, i.e. uniform on [-init_scale, init_scale).
inline uint64_t splitmix_out(uint64_t seed, uint64_t nth /*1-based*/) {
    uint64_t z = seed + nth * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
inline float init_value(uint64_t key, int j, float init_scale, int dtype) {
    uint64_t z = splitmix_out(key, static_cast<uint64_t>(j) + 1ull);
    int32_t q = static_cast<int32_t>(z >> 40) - (1 << 23);
    double c = static_cast<double>(init_scale) * (1.0 / 8388608.0); // exact power-of-two scaling
    float v = static_cast<float>(static_cast<double>(q) * c);     // one rounding, as one fp32 multiply
    if (dtype == kBF16) v = bf16_bits_to_float(float_to_bf16_bits(v));
    return v;
}

Row fresh_row(const Table& t, uint64_t key) {
    Row r;
    r.w.resize(t.dim);
    for (int j = 0; j < t.dim; ++j) r.w[j] = init_value(key, j, t.init_scale, t.dtype);
    return r;
}

inline bool key_ok(uint64_t k) { return (k >> 63) == 0; }

// What a lookup delivers for element j of a row: the stored value, a hot row's fp32 master
// rounded to the table's 16-bit type (App. C "Mixed Precision Training").
inline float delivered(const Row& r, int j) {
    return r.hot ? bf16_bits_to_float(float_to_bf16_bits(r.w[j])) : r.w[j];
}

} // namespace

extern "C" {

// ---------------------------------------------------------------------------
// Table merging (Sec. 3.2 "Automated Merging Table"): logical tables with the
// same (dim, dtype) share one hash table.  Merged tables are numbered in order
// of first appearance.  Returns the number of merged tables.
int orc_plan_merge(const int* dims, const int* dtypes, int m, int* merged_of) {
    std::vector<std::pair<int, int>> seen;
    for (int t = 0; t < m; ++t) {
        std::pair<int, int> sig(dims[t], dtypes[t]);
        auto it = std::find(seen.begin(), seen.end(), sig);
        if (it == seen.end()) {
            seen.push_back(sig);
            merged_of[t] = static_cast<int>(seen.size()) - 1;
        } else {
            merged_of[t] = static_cast<int>(it - seen.begin());
        }
    }
    return static_cast<int>(seen.size());
}

// Number of identifier bits for m tables: k = ceil(log2(m + 1))  (Sec. 3.2).
int orc_tag_bits(int m) {
    int k = 0;
    while ((1ll << k) < static_cast<long long>(m) + 1) ++k;
    return k;
}

// Eq. 8: ID = (i << (63 - k)) | x, top bit zero.  Element e belongs to the
// field f with field_off[f] <= e < field_off[f+1]; field_tag[f] is the
// 0-based logical table index i.  A raw ID that does not fit in 63-k bits is
// counted in *err_count and wrapped into range (x mod 2^(63-k)).
int orc_tag_keys(const uint64_t* x, const int64_t* field_off, const uint8_t* field_tag, int n_fields,
                 int tag_bits, uint64_t* key_out, int64_t* err_count) {
    if (tag_bits < 0 || tag_bits > 16) return -1;
    const int shift = 63 - tag_bits;
    const uint64_t low_mask = (1ull << shift) - 1ull;
    int64_t errs = 0;
    for (int f = 0; f < n_fields; ++f) {
        if (tag_bits < 8 && (field_tag[f] >> tag_bits) != 0) return -1; // table index needs more than k bits
        for (int64_t e = field_off[f]; e < field_off[f + 1]; ++e) {
            uint64_t v = x[e];
            if (v > low_mask) { ++errs; v &= low_mask; }
            key_out[e] = (static_cast<uint64_t>(field_tag[f]) << shift) | v;
        }
    }
    if (err_count) *err_count = errs;
    return 0;
}

// ---------------------------------------------------------------------------
// Deduplication (Sec. 3.3): the distinct keys in ascending order, for every
// input position the index of its key among them, and how often each occurs.
int64_t orc_dedup(const uint64_t* key, int64_t n, uint64_t* uniq, int32_t* inverse, int32_t* counts) {
    std::vector<uint64_t> s(key, key + n);
    std::sort(s.begin(), s.end());
    s.erase(std::unique(s.begin(), s.end()), s.end());
    const int64_t U = static_cast<int64_t>(s.size());
    for (int64_t u = 0; u < U; ++u) {
        uniq[u] = s[u];
        if (counts) counts[u] = 0;
    }
    for (int64_t i = 0; i < n; ++i) {
        int64_t u = std::lower_bound(s.begin(), s.end(), key[i]) - s.begin();
        inverse[i] = static_cast<int32_t>(u);
        if (counts) ++counts[u];
    }
    return U;
}

// ---------------------------------------------------------------------------
// Dynamic table (Sec. 3.1).
void* orc_table_create(int dim, int dtype, float init_scale) {
    if (dim <= 0 || (dtype != kF32 && dtype != kBF16)) return nullptr;
    Table* t = new Table();
    t->dim = dim;
    t->dtype = dtype;
    t->init_scale = init_scale;
    return t;
}
void orc_table_destroy(void* h) { delete static_cast<Table*>(h); }
int64_t orc_size(void* h) { return static_cast<int64_t>(static_cast<Table*>(h)->map.size()); }

// Closed-form initial row of a key (what a never-updated row must equal).
void orc_init_row(uint64_t key, int dim, int dtype, float init_scale, float* out) {
    for (int j = 0; j < dim; ++j) out[j] = init_value(key, j, init_scale, dtype);
}

// Find each key; an absent key is inserted with its initial row, acc = 0,
// freq = 0.  Then every element (duplicates included) counts one touch:
// freq += 1, last_seen = step.  inserted[i] = 1 for the element that created
// the entry.  Keys with the top bit set are rejected (return -2, nothing done).
int orc_find_or_insert(void* h, const uint64_t* key, int64_t n, uint32_t step, uint8_t* inserted) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i)
        if (!key_ok(key[i])) return -2;
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        bool created = false;
        if (it == t.map.end()) {
            it = t.map.emplace(key[i], fresh_row(t, key[i])).first;
            created = true;
        }
        it->second.freq += 1;
        it->second.last_seen = step;
        if (inserted) inserted[i] = created ? 1 : 0;
    }
    return 0;
}

// Bulk-load semantics for keys that exist before the first step: identical to
// one find-or-insert touch at step 0, applied only to keys not yet present
// (so calling it again, or lazily for the keys a step is about to touch, is
// harmless).
int orc_prepopulate(void* h, const uint64_t* key, int64_t n) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i) {
        if (!key_ok(key[i])) return -2;
        if (t.map.find(key[i]) == t.map.end()) {
            Row r = fresh_row(t, key[i]);
            r.freq = 1;
            r.last_seen = 0;
            t.map.emplace(key[i], std::move(r));
        }
    }
    return 0;
}

// Read-only membership.
int orc_find(void* h, const uint64_t* key, int64_t n, uint8_t* found) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i) found[i] = t.map.count(key[i]) ? 1 : 0;
    return 0;
}

// Rows of the given keys as float32 [n, dim]; an absent key reads as zeros.
int orc_lookup(void* h, const uint64_t* key, int64_t n, float* out) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        float* o = out + i * t.dim;
        if (it == t.map.end()) {
            for (int j = 0; j < t.dim; ++j) o[j] = 0.0f;
        } else {
            for (int j = 0; j < t.dim; ++j) o[j] = delivered(it->second, j);
        }
    }
    return 0;
}

// The forward pass by its plain definition, without deduplication: every
// position looks its key up directly; absent keys are created on the spot.
// Touch counters are left alone (freq = 0 for rows created here).
int orc_direct_lookup(void* h, const uint64_t* key, int64_t n, uint32_t step, float* out) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i) {
        if (!key_ok(key[i])) return -2;
        auto it = t.map.find(key[i]);
        if (it == t.map.end()) {
            Row r = fresh_row(t, key[i]);
            r.last_seen = step;
            it = t.map.emplace(key[i], std::move(r)).first;
        }
        for (int j = 0; j < t.dim; ++j) out[i * t.dim + j] = delivered(it->second, j);
    }
    return 0;
}

// Expand: E[i,:] = E_u[inverse[i],:]  (undoes the deduplication).
int orc_expand(const float* uniq_rows, const int32_t* inverse, int64_t n, int dim, float* out) {
    for (int64_t i = 0; i < n; ++i)
        for (int j = 0; j < dim; ++j) out[i * dim + j] = uniq_rows[static_cast<int64_t>(inverse[i]) * dim + j];
    return 0;
}

// Gradient aggregation per distinct key: g[u,:] = sum over positions i with
// inverse[i] == u of G[i,:], accumulated in double in input order and rounded
// once to float.
int orc_segment_reduce(const float* grad, const int32_t* inverse, int64_t n, int64_t n_unique, int dim,
                       float* reduced) {
    std::vector<double> sum(static_cast<size_t>(n_unique) * dim, 0.0);
    for (int64_t i = 0; i < n; ++i) {
        int64_t u = inverse[i];
        if (u < 0 || u >= n_unique) return -1;
        for (int j = 0; j < dim; ++j) sum[u * dim + j] += static_cast<double>(grad[i * dim + j]);
    }
    for (size_t e = 0; e < sum.size(); ++e) reduced[e] = static_cast<float>(sum[e]);
    return 0;
}

// Pooling of bags (Sec. 3.2: the table collection "performs pooling computations as needed").
// Bag b is the run of positions bag_off[b] .. bag_off[b+1]-1.  pooled[b,:] = sum (or mean) of the
// rows E[i,:] of its positions, accumulated in double in position order, rounded once.  An empty
// bag gives zeros.
int orc_pool_bags(const float* E, const int64_t* bag_off, int64_t n_bags, int dim, int mean, float* pooled) {
    for (int64_t b = 0; b < n_bags; ++b) {
        const int64_t len = bag_off[b + 1] - bag_off[b];
        if (len < 0) return -1;
        for (int j = 0; j < dim; ++j) {
            double s = 0.0;
            for (int64_t i = bag_off[b]; i < bag_off[b + 1]; ++i) s += static_cast<double>(E[i * dim + j]);
            if (mean && len > 0) s /= static_cast<double>(len);
            pooled[b * dim + j] = static_cast<float>(s);
        }
    }
    return 0;
}

// Backward of the pooling: the gradient of position i is the gradient of its bag's pooled vector,
// divided by the bag length for the mean (one correctly rounded fp32 division).
int orc_pool_bags_backward(const float* d_pooled, const int64_t* bag_off, int64_t n_bags, int dim, int mean, float* G) {
    for (int64_t b = 0; b < n_bags; ++b) {
        const int64_t len = bag_off[b + 1] - bag_off[b];
        for (int64_t i = bag_off[b]; i < bag_off[b + 1]; ++i)
            for (int j = 0; j < dim; ++j) {
                const float g = d_pooled[b * dim + j];
                G[i * dim + j] = mean ? g / static_cast<float>(len) : g;
            }
    }
    return 0;
}

// Row-wise Adagrad on the rows of the given keys only:
//   acc <- acc + (1/D) * sum_j g_j^2 ;  w_j <- w_j - lr * g_j / (sqrt(acc) + eps)
// evaluated in double from the stored state, each stored value rounded once.
// Absent keys are skipped.  A key listed twice is updated twice, in order.
int orc_apply_adagrad(void* h, const uint64_t* key, int64_t n, const float* g, float lr, float eps) {
    Table& t = *static_cast<Table*>(h);
    const int D = t.dim;
    for (int64_t u = 0; u < n; ++u) {
        auto it = t.map.find(key[u]);
        if (it == t.map.end()) continue;
        Row& r = it->second;
        double ss = 0.0;
        for (int j = 0; j < D; ++j) ss += static_cast<double>(g[u * D + j]) * static_cast<double>(g[u * D + j]);
        double acc = static_cast<double>(r.acc) + ss / static_cast<double>(D);
        double denom = std::sqrt(acc) + static_cast<double>(eps);
        for (int j = 0; j < D; ++j) {
            double w = static_cast<double>(r.w[j]) - static_cast<double>(lr) * static_cast<double>(g[u * D + j]) / denom;
            r.w[j] = (t.dtype == kBF16 && !r.hot) ? double_to_bf16_float(w) : static_cast<float>(w);
        }
        r.acc = static_cast<float>(acc);
    }
    return 0;
}

// Sparse (lazy) Adam on the rows of the given keys only, the optimizer of Sec. 4.1:
//   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
//   w <- w - lr * sqrt(1-b2^t)/(1-b1^t) * m / (sqrt(v) + eps)
// evaluated in double from the stored fp32 state; m, v, w each rounded once on store.  Absent keys
// are skipped.  A new entry starts with zero moments.
int orc_apply_adam(void* h, const uint64_t* key, int64_t n, const float* g, float lr, float b1, float b2, float eps,
                   int64_t step) {
    Table& t = *static_cast<Table*>(h);
    const int D = t.dim;
    if (step < 1) return -1;
    const double B1 = b1, B2 = b2;
    const double step_size = static_cast<double>(lr) * std::sqrt(1.0 - std::pow(B2, (double)step)) / (1.0 - std::pow(B1, (double)step));
    for (int64_t u = 0; u < n; ++u) {
        auto it = t.map.find(key[u]);
        if (it == t.map.end()) continue;
        Row& r = it->second;
        if (r.m.empty()) {
            r.m.assign(D, 0.0f);
            r.v.assign(D, 0.0f);
        }
        for (int j = 0; j < D; ++j) {
            const double gg = g[u * D + j];
            const double m = B1 * (double)r.m[j] + (1.0 - B1) * gg;
            const double v = B2 * (double)r.v[j] + (1.0 - B2) * gg * gg;
            const double w = (double)r.w[j] - step_size * m / (std::sqrt(v) + (double)eps);
            r.m[j] = static_cast<float>(m);
            r.v[j] = static_cast<float>(v);
            r.w[j] = (t.dtype == kBF16 && !r.hot) ? double_to_bf16_float(w) : static_cast<float>(w);   // a master stays fp32
        }
    }
    return 0;
}

// Eviction at step `now`.  A key goes when it has not been touched for `ttl`
// steps (rule active when ttl > 0), or when it was touched fewer than
// `min_freq` times and not within the last `grace` steps (rule active when
// min_freq > 0).  The erased keys are written in ascending order; returns how
// many.  evicted may be null.
int64_t orc_evict(void* h, uint32_t now, uint32_t ttl, uint32_t min_freq, uint32_t grace, uint64_t* evicted) {
    Table& t = *static_cast<Table*>(h);
    std::vector<uint64_t> gone;
    for (const auto& kv : t.map) {
        uint32_t age = now - kv.second.last_seen;
        bool stale = (ttl > 0) && (age >= ttl);
        bool rare = (min_freq > 0) && (kv.second.freq < min_freq) && (age >= grace);
        if (stale || rare) gone.push_back(kv.first);
    }
    std::sort(gone.begin(), gone.end());
    for (uint64_t k : gone) {
        if (t.map.at(k).hot) t.hot_used -= 1; // its master goes back to the hot store
        t.map.erase(k);
    }
    if (evicted) std::copy(gone.begin(), gone.end(), evicted);
    return static_cast<int64_t>(gone.size());
}

// Dump of the whole table ordered by key (values as float32).  Any output may
// be null.  Returns the number of entries.
int64_t orc_export(void* h, uint64_t* keys, float* values, float* acc, uint32_t* last_seen, uint32_t* freq) {
    Table& t = *static_cast<Table*>(h);
    std::vector<uint64_t> ks;
    ks.reserve(t.map.size());
    for (const auto& kv : t.map) ks.push_back(kv.first);
    std::sort(ks.begin(), ks.end());
    for (size_t i = 0; i < ks.size(); ++i) {
        const Row& r = t.map.at(ks[i]);
        if (keys) keys[i] = ks[i];
        if (values) for (int j = 0; j < t.dim; ++j) values[i * t.dim + j] = delivered(r, j);
        if (acc) acc[i] = r.acc;
        if (last_seen) last_seen[i] = r.last_seen;
        if (freq) freq[i] = r.freq;
    }
    return static_cast<int64_t>(ks.size());
}

// State of the given keys (for sampled comparisons on large tables).
// present[i] = 0 leaves the other outputs of that entry untouched.
int orc_peek(void* h, const uint64_t* key, int64_t n, uint8_t* present, float* values, float* acc,
             uint32_t* last_seen, uint32_t* freq) {
    Table& t = *static_cast<Table*>(h);
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        present[i] = it != t.map.end();
        if (!present[i]) continue;
        const Row& r = it->second;
        if (values) for (int j = 0; j < t.dim; ++j) values[i * t.dim + j] = delivered(r, j);
        if (acc) acc[i] = r.acc;
        if (last_seen) last_seen[i] = r.last_seen;
        if (freq) freq[i] = r.freq;
    }
    return 0;
}

// ---- hot / cold rows (App. C "Mixed Precision Training") --------------------
// Frequently used keys of a 16-bit table keep their vector in fp32; the rest stay 16-bit.
// The hot store holds at most `capacity` masters.
int orc_set_hot(void* h, int64_t capacity) {
    Table& t = *static_cast<Table*>(h);
    if (t.dtype != kBF16 || capacity <= 0) return -1;
    t.hot_capacity = capacity;
    return 0;
}
// Promote, in the order given, every present key touched at least min_freq times that is not
// hot yet, while the hot store has room.  The master starts as the row's current 16-bit values.
// Returns how many were promoted.
int64_t orc_promote(void* h, const uint64_t* key, int64_t n, uint32_t min_freq) {
    Table& t = *static_cast<Table*>(h);
    int64_t done = 0;
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        if (it == t.map.end()) continue;
        Row& r = it->second;
        if (r.hot || r.freq < min_freq || t.hot_used >= t.hot_capacity) continue;
        r.hot = true;
        t.hot_used += 1;
        done += 1;
    }
    return done;
}
// Demote: the partition into hot and cold keys follows the access pattern both ways (App. C: hot sets are
// partitioned dynamically).  Every hot row that no lookup has touched for `idle` steps (now - last_seen >= idle)
// gives its master back to the hot store: the 16-bit row becomes the master rounded to nearest even - which is
// what lookups delivered for it anyway - and later updates round as for any cold row.  Returns how many.
int64_t orc_demote(void* h, uint32_t now, uint32_t idle) {
    Table& t = *static_cast<Table*>(h);
    int64_t done = 0;
    for (auto& kv : t.map) {
        Row& r = kv.second;
        if (!r.hot || now - r.last_seen < idle) continue;
        for (int j = 0; j < t.dim; ++j) r.w[j] = bf16_bits_to_float(float_to_bf16_bits(r.w[j]));
        r.hot = false;
        t.hot_used -= 1;
        done += 1;
    }
    return done;
}
// Restore dumped entries (App. C "Checkpoint Resuming"): every listed key that is present takes the dumped row
// (values[i,:] as a lookup delivered it; exact for a 16-bit table since the dump holds 16-bit values), accumulator,
// last-seen step and touch count.  A hot row's master follows the row.  Returns how many keys were present.
int64_t orc_put(void* h, const uint64_t* key, int64_t n, const float* values, const float* acc,
                const uint32_t* last_seen, const uint32_t* freq) {
    Table& t = *static_cast<Table*>(h);
    int64_t done = 0;
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        if (it == t.map.end()) continue;
        Row& r = it->second;
        if (values) for (int j = 0; j < t.dim; ++j) r.w[j] = values[i * t.dim + j];
        if (acc) r.acc = acc[i];
        if (last_seen) r.last_seen = last_seen[i];
        if (freq) r.freq = freq[i];
        done += 1;
    }
    return done;
}
// Restore masters from a dump (App. C "Checkpoint Resuming" for a table with hot rows): the master of every listed
// key that is present and hot becomes values[i,:] (fp32, as ht_export_hot / orc_export_hot wrote it); keys that are
// absent or cold are skipped.  Returns how many masters were written.
int64_t orc_put_hot(void* h, const uint64_t* key, int64_t n, const float* values) {
    Table& t = *static_cast<Table*>(h);
    int64_t done = 0;
    for (int64_t i = 0; i < n; ++i) {
        auto it = t.map.find(key[i]);
        if (it == t.map.end() || !it->second.hot) continue;
        for (int j = 0; j < t.dim; ++j) it->second.w[j] = values[i * t.dim + j];
        done += 1;
    }
    return done;
}
// Masters ordered by key: keys[n_hot], values[n_hot, dim] (either may be null).  Returns n_hot.
int64_t orc_export_hot(void* h, uint64_t* keys, float* values) {
    Table& t = *static_cast<Table*>(h);
    std::vector<uint64_t> ks;
    for (const auto& kv : t.map) if (kv.second.hot) ks.push_back(kv.first);
    std::sort(ks.begin(), ks.end());
    for (size_t i = 0; i < ks.size(); ++i) {
        if (keys) keys[i] = ks[i];
        if (values) std::copy(t.map.at(ks[i]).w.begin(), t.map.at(ks[i]).w.end(), values + i * t.dim);
    }
    return static_cast<int64_t>(ks.size());
}

// bf16 helpers exposed for the tests' own cross-checks.
void orc_float_to_bf16(const float* in, int64_t n, uint16_t* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = float_to_bf16_bits(in[i]);
}
void orc_bf16_to_float(const uint16_t* in, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_bits_to_float(in[i]);
}

} // extern "C"
