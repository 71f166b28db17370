// CPU oracle for the collisionless embedding table hot path.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, sequential model of what the
// device library must compute.  Only the test-suite, the smoke check and the CPU-baseline leg
// of the benchmark may load it; the product path never does, and the two share no code.
//
// Two independent models live here behind one C interface:
//
//   kind 0  "R0"  the definition written out: an ordered map key -> {row, accumulator,
//                 last-seen step} of unbounded size, plus an ordered map for the occurrence
//                 counters.  No hashing of table positions at all.
//   kind 1  "R1"  the oracle proper: the cuckoo hashmap of the paper's section 2.1 (two
//                 sub-tables T0/T1 with hash functions h0/h1, insertion by eviction chain),
//                 taken in the paper's order: try T0[h0(A)], if occupied evict the occupant B,
//                 put A there, and insert B into the other sub-table by the same procedure.
//
// Both implement the same batch semantics (section 2.1's admission filter and expiry, plus the
// pooling / gradient reduction / Adagrad steps that the build's problem statement adds):
//   1. occurrences are split into hits and misses against the table as it was BEFORE the batch;
//   2. every miss occurrence bumps its key's occurrence counter (saturating at 255);
//   3. every distinct missing key whose counter is now >= freq_threshold is admitted with a
//      row that is a pure function of (seed, key), accumulator 0 and last_seen = step - unless
//      that would take the table past its fill limit of capacity - capacity/32 keys: then none
//      of the batch's new keys is admitted (the rule does not depend on any order of the keys);
//   4. every hit key gets last_seen = step;
//   5. an occurrence is "present" iff its key is in the table after step 3;
//   6. pooling sums the rows of the present occurrences of each bag (fp64 accumulate);
//   7. the gradient of a key is the fp64 sum of the pooled gradients of the bags holding it,
//      once per occurrence;
//   8. row-wise Adagrad is applied once per distinct key: acc += mean_j g_j^2,
//      w_j -= lr * g_j / (sqrt(acc) + eps);
//   9. sweep(now) erases every key with now - last_seen >= expire_steps (expire_steps > 0).
//
// Three maintenance operations around that path (same two models, same interface):
//  10. touched keys (the paper's incremental parameter synchronisation): the set of keys whose
//      embeddings were trained since the last synchronisation; taking it clears it; a key that
//      expires leaves it;
//  11. snapshot / restore (the paper's fault tolerance): the dump plus the counter words are the
//      snapshot; restore places given (key, row, accumulator, last-seen) records into a table
//      and writes counter words back;
//  12. rehash / grow (section 2.1: rehash when an insertion runs into a cycle): every stored key
//      is re-inserted under the hash functions of a new generation, in a table of the same or a
//      larger power-of-two capacity; when the number of counters grows by 2^k, a counter's value
//      goes to all 2^k counters that its keys can now map to (never an under-count).
//
// Beside the table: the paper's hashing baseline (section 3.1, the production model's tables), the
// quotient-remainder decomposition, as a pooling routine over two dense tables:
//  13. ID_r = ID mod 2^m, ID_q = ID div 2^m, E = E_r[ID_r] + E_q[ID_q]; a bag's output is the fp64
//      sum of E over its IDs, rounded once; an ID outside [0, 2^(2m)) contributes nothing.
//
// Parity unpinned: what happens when an eviction chain exceeds its bound (which key ends up in
// the overflow stash depends on insertion order); graded runs must have zero such failures.
//
// Build: g++ -O2 -std=c++17 -shared -fPIC monolith_oracle.cpp -o libmonolith_oracle.so

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <map>
#include <memory>
#include <set>
#include <vector>

namespace {

constexpr uint64_t kEmptyKey = ~0ull;  // reserved key: padding, never stored

// ---------------------------------------------------------------------------------------------
// Hashing.  The paper only asks for two different hash functions h0, h1 (section 2.1); this build
// fixes one public 64-bit mixer (the SplitMix64 output function) and derives every hash from it.
// ---------------------------------------------------------------------------------------------
uint64_t mix64(uint64_t z) {
  z ^= z >> 30;
  z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27;
  z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

// salt i is the (i+1)-th output of the SplitMix64 generator started at `seed`.
uint64_t salt(uint64_t seed, int i) { return mix64(seed + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull); }
// The placement hashes h0 / h1 of rehash generation g use the salts of seed + g * (an odd
// constant); generation 0 is the table as created.  Counter and initial-value hashes never change.
uint64_t placement_seed(uint64_t seed, uint32_t generation) {
  return seed + (uint64_t)generation * 0xD1B54A32D192ED03ull;
}

// top `lg` bits of h (0 when lg == 0)
uint64_t top_bits(uint64_t h, int lg) { return lg == 0 ? 0 : h >> (64 - lg); }

int log2_exact(uint64_t v) {
  int lg = 0;
  while ((1ull << lg) < v) ++lg;
  return lg;
}

// Initial embedding value: uniform on a 2^-27 grid in [-2^-4, 2^-4).  Every operation is exact
// in fp32 (24-bit integer -> float, power-of-two scaling, one subtraction of 1).
float init_value(uint64_t s_init, uint64_t key, uint32_t j) {
  uint64_t h = mix64(mix64(key ^ s_init) + (uint64_t)j);
  uint32_t u24 = (uint32_t)(h >> 40);
  return ((float)u24 * (1.0f / 8388608.0f) - 1.0f) * 0.0625f;
}

// bfloat16 storage: round to nearest, ties to even, on the fp32 bit pattern.
float bf16_round(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u) {  // inf / nan: truncate, keep nan a nan
    if (u & 0x007FFFFFu) u |= 0x00400000u;
    u &= 0xFFFF0000u;
  } else {
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
  }
  float y;
  std::memcpy(&y, &u, 4);
  return y;
}

struct Params {
  uint64_t capacity = 0;   // total slots = rows (R1); R0 ignores it except for the filter size
  uint32_t dim = 0;
  uint64_t seed = 0;
  uint32_t freq_threshold = 0;  // 0 and 1 both admit on first sight; <= 255
  uint32_t expire_steps = 0;    // 0 = never
  bool bf16 = false;            // rows stored in bfloat16
  uint64_t n_filter = 0;        // number of occurrence counters (power of two)
  int lg_filter = 0;
  uint32_t filter_hashes = 1;   // counters per key (1..4): the key's count is the MINIMUM of them
  uint64_t s_h0 = 0, s_h1 = 0, s_init = 0;
  uint64_t s_filter[4] = {0, 0, 0, 0};
};

// Occurrence counter word, canonical form: (step & 0xFFFFFF) << 8 | count, count saturates at
// 255.  A word that was last touched expire_steps or more steps ago restarts from zero at its
// next touch (expire_steps == 0: never).
uint32_t filter_touch(uint32_t word, uint32_t step, uint32_t expire_steps) {
  uint32_t last = word >> 8, count = word & 255u;
  if (expire_steps > 0 && step - last >= expire_steps) count = 0;
  if (count < 255u) ++count;
  return (step << 8) | count;
}

struct Entry {
  std::vector<float> w;  // dim values (already rounded to the storage type)
  float acc = 0.0f;
  uint32_t last_seen = 0;
};

void init_entry(const Params& p, uint64_t key, uint32_t step, Entry* e) {
  e->w.resize(p.dim);
  for (uint32_t j = 0; j < p.dim; ++j) {
    float v = init_value(p.s_init, key, j);
    e->w[j] = p.bf16 ? bf16_round(v) : v;
  }
  e->acc = 0.0f;
  e->last_seen = step;
}

// Row-wise Adagrad on one entry with the already reduced gradient g (fp64).
void adagrad_entry(const Params& p, const std::vector<double>& g, double lr, double eps, Entry* e) {
  double ss = 0.0;
  for (uint32_t j = 0; j < p.dim; ++j) ss += g[j] * g[j];
  double acc = (double)e->acc + ss / (double)p.dim;
  double denom = std::sqrt(acc) + eps;
  for (uint32_t j = 0; j < p.dim; ++j) {
    float v = (float)((double)e->w[j] - lr * g[j] / denom);
    e->w[j] = p.bf16 ? bf16_round(v) : v;
  }
  e->acc = (float)acc;
}

struct Exported {
  uint64_t key;
  const Entry* e;
  int64_t slot;  // global slot index (R1), -1 for "no position" (R0) and -2 for the stash
};

class Model {
 public:
  explicit Model(const Params& p) : p_(p) {}
  virtual ~Model() = default;
  virtual void lookup_or_insert(const int64_t* keys, uint64_t n, uint32_t step, uint8_t* present) = 0;
  virtual void pool(const int64_t* keys, const int64_t* offsets, uint64_t n_bags, float* out) = 0;
  virtual void apply_grad(const int64_t* keys, const int64_t* offsets, uint64_t n_bags,
                          const float* grad, float lr, float eps) = 0;
  virtual void sweep(uint32_t now, std::vector<uint64_t>* erased) = 0;
  virtual void dump(std::vector<Exported>* out) const = 0;  // sorted by key
  virtual uint32_t filter_word(uint64_t index) const = 0;
  // -- maintenance ------------------------------------------------------------------------------
  // keys trained since the last call, ascending; the set is cleared
  void take_touched(std::vector<uint64_t>* out) {
    out->assign(touched_.begin(), touched_.end());
    touched_.clear();
  }
  // place a record; false (and nothing changes) if the key is already stored or is the reserved key.
  // Where counters never age (expire_steps == 0) a stored key's counters are at or above the admission
  // threshold at all times, so a placed key's counters are raised to it if they are below (records may be
  // restored without their counters).  Where counters age there is no such invariant - the counter of a
  // stored key may have restarted since - and a restore must give back the snapshot as it was: nothing is raised.
  virtual bool import_entry(uint64_t key, const Entry& e) = 0;
  virtual bool is_stored(uint64_t key) const = 0;
  virtual uint64_t size() const = 0;
  void count_refused_full(uint64_t n) { refused_full_ += n; }
  void raise_counters(uint64_t key) {
    if (p_.expire_steps != 0) return;
    uint32_t least = p_.freq_threshold > 1 ? p_.freq_threshold : 1;
    for (uint32_t j = 0; j < p_.filter_hashes; ++j) {
      uint64_t i = filter_index(key, j);
      uint32_t w = filter_word(i);
      if ((w & 255u) < least) set_filter_word(i, (w & ~255u) | least);
    }
  }
  virtual void set_filter_word(uint64_t index, uint32_t word) = 0;
  // Counter words [first, first + count) are replaced (restore of the counters of a snapshot).  Where
  // counters never age a stored key stays counted: any of its counters among the written ones that is
  // now below the admission threshold is raised to it, exactly as when a record is restored without
  // its counters (for the words of a consistent snapshot that changes nothing).
  void write_filter_words(uint64_t first, uint64_t count, const uint32_t* words) {
    for (uint64_t i = 0; i < count; ++i) set_filter_word(first + i, words[i]);
    if (p_.expire_steps != 0) return;
    std::vector<Exported> stored;
    dump(&stored);
    uint32_t least = p_.freq_threshold > 1 ? p_.freq_threshold : 1;
    for (const Exported& x : stored)
      for (uint32_t j = 0; j < p_.filter_hashes; ++j) {
        uint64_t i = filter_index(x.key, j);
        if (i < first || i - first >= count) continue;
        uint32_t w = filter_word(i);
        if ((w & 255u) < least) set_filter_word(i, (w & ~255u) | least);
      }
  }
  // re-insert everything under generation `generation` in a table of `new_capacity` >= capacity
  virtual void rehash(uint64_t new_capacity, uint32_t generation) = 0;
  virtual uint64_t insert_failures() const { return 0; }
  virtual uint64_t max_chain() const { return 0; }
  const Params& params() const { return p_; }
  // Fill limit: a table of `capacity` slots stores at most capacity - capacity/32 keys (with buckets of
  // eight, eviction chains grow steeply beyond that load).  A call whose new keys would take the table
  // past the limit places NONE of them (whatever their order); they are counted as refused.
  uint64_t fill_limit() const { return p_.capacity - p_.capacity / 32; }
  uint64_t refused_full() const { return refused_full_; }
  // counter j of a key (j < filter_hashes); every hash addresses the whole array
  uint64_t filter_index(uint64_t key, uint32_t j = 0) const {
    return top_bits(mix64(key ^ p_.s_filter[j]), p_.lg_filter);
  }

 protected:
  // new table geometry and placement salts; returns log2 of the growth factor of the counter array
  int regrow_params(uint64_t new_capacity, uint32_t generation) {
    int k = log2_exact(new_capacity / p_.capacity);
    p_.capacity = new_capacity;
    p_.n_filter <<= k;
    p_.lg_filter += k;
    p_.s_h0 = salt(placement_seed(p_.seed, generation), 0);
    p_.s_h1 = salt(placement_seed(p_.seed, generation), 1);
    return k;
  }
  Params p_;
  std::set<uint64_t> touched_;
  uint64_t refused_full_ = 0;
};

// ---------------------------------------------------------------------------------------------
// R0: the definition.  std::map everywhere, nothing clever.
// ---------------------------------------------------------------------------------------------
class BruteForceModel final : public Model {
 public:
  using Model::Model;

  void lookup_or_insert(const int64_t* keys, uint64_t n, uint32_t step, uint8_t* present) override {
    std::vector<uint8_t> was_hit(n, 0);
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey) continue;
      was_hit[i] = table_.count(k) ? 1 : 0;
    }
    // all counting first ...
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey || was_hit[i]) continue;
      for (uint32_t j = 0; j < p_.filter_hashes; ++j) {  // one touch per counter of the key
        uint32_t& w = filter_[filter_index(k, j)];
        w = filter_touch(w, step, p_.expire_steps);
      }
    }
    // ... then admission: the key's count is the smallest of its counters
    std::set<uint64_t> admissible;
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey || was_hit[i]) continue;
      uint32_t count = 255u;
      for (uint32_t j = 0; j < p_.filter_hashes; ++j) count = std::min(count, filter_[filter_index(k, j)] & 255u);
      if (count >= p_.freq_threshold) admissible.insert(k);
    }
    if (table_.size() + admissible.size() > fill_limit()) {
      refused_full_ += admissible.size();  // the batch would overfill the table: none of its new keys gets in
    } else {
      for (uint64_t k : admissible) init_entry(p_, k, step, &table_[k]);
    }
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey) { present[i] = 0; continue; }
      auto it = table_.find(k);
      if (it != table_.end() && was_hit[i]) it->second.last_seen = step;
      present[i] = it != table_.end();
    }
  }

  void pool(const int64_t* keys, const int64_t* offsets, uint64_t n_bags, float* out) override {
    std::vector<double> s(p_.dim);
    for (uint64_t b = 0; b < n_bags; ++b) {
      std::fill(s.begin(), s.end(), 0.0);
      for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
        auto it = table_.find((uint64_t)keys[i]);
        if (it == table_.end()) continue;
        for (uint32_t j = 0; j < p_.dim; ++j) s[j] += (double)it->second.w[j];
      }
      for (uint32_t j = 0; j < p_.dim; ++j) out[b * p_.dim + j] = (float)s[j];
    }
  }

  void apply_grad(const int64_t* keys, const int64_t* offsets, uint64_t n_bags, const float* grad,
                  float lr, float eps) override {
    std::map<uint64_t, std::vector<double>> g;
    for (uint64_t b = 0; b < n_bags; ++b)
      for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
        uint64_t k = (uint64_t)keys[i];
        if (!table_.count(k)) continue;
        std::vector<double>& gk = g[k];
        gk.resize(p_.dim, 0.0);
        for (uint32_t j = 0; j < p_.dim; ++j) gk[j] += (double)grad[b * p_.dim + j];
      }
    for (auto& kv : g) {
      adagrad_entry(p_, kv.second, (double)lr, (double)eps, &table_[kv.first]);
      touched_.insert(kv.first);
    }
  }

  void sweep(uint32_t now, std::vector<uint64_t>* erased) override {
    erased->clear();
    if (p_.expire_steps == 0) return;
    for (auto it = table_.begin(); it != table_.end();) {
      if (now - it->second.last_seen >= p_.expire_steps) {
        erased->push_back(it->first);
        touched_.erase(it->first);
        it = table_.erase(it);
      } else {
        ++it;
      }
    }
  }

  void dump(std::vector<Exported>* out) const override {
    out->clear();
    for (auto& kv : table_) out->push_back({kv.first, &kv.second, -1});
  }

  uint32_t filter_word(uint64_t index) const override {
    auto it = filter_.find(index);
    return it == filter_.end() ? 0u : it->second;
  }

  bool import_entry(uint64_t key, const Entry& e) override {
    if (key == kEmptyKey || table_.count(key)) return false;
    table_[key] = e;
    raise_counters(key);
    return true;
  }
  bool is_stored(uint64_t key) const override { return table_.count(key) != 0; }
  uint64_t size() const override { return table_.size(); }
  void set_filter_word(uint64_t index, uint32_t word) override { filter_[index] = word; }
  void rehash(uint64_t new_capacity, uint32_t generation) override {
    int k = regrow_params(new_capacity, generation);  // the map itself has no positions to redo
    std::map<uint64_t, uint32_t> grown;
    for (auto& iw : filter_)
      for (uint64_t c = 0; c < (1ull << k); ++c) grown[(iw.first << k) + c] = iw.second;
    filter_.swap(grown);
  }

 private:
  std::map<uint64_t, Entry> table_;
  std::map<uint64_t, uint32_t> filter_;
};

// ---------------------------------------------------------------------------------------------
// R1: cuckoo hashmap as described in section 2.1 of the paper.
//
// Sub-table T_i has capacity/2 slots grouped into buckets of `bucket` slots; an element x may only
// live in bucket h_i(x) of T_i.  bucket == 1 is the textbook structure the paper describes; a
// wider bucket is the usual generalisation that lets the load factor go past 0.5.  A slot stores
// the key and the index of its entry in a side pool, so an eviction moves 12 bytes, not a row.
//
// hash_mode 1 replaces the mixer by a toy pair (h0 = k mod m, h1 = (k div m) mod m, m = buckets
// per sub-table) so that a placement can be traced by hand.
// ---------------------------------------------------------------------------------------------
class CuckooModel final : public Model {
 public:
  CuckooModel(const Params& p, uint32_t bucket, uint32_t max_kicks, int hash_mode)
      : Model(p), bucket_(bucket), max_kicks_(max_kicks), hash_mode_(hash_mode) {
    n_buckets_ = p.capacity / 2 / bucket;  // per sub-table
    lg_buckets_ = log2_exact(n_buckets_);
    slot_key_.assign(p.capacity, kEmptyKey);
    slot_entry_.assign(p.capacity, -1);
    filter_.assign(p.n_filter, 0u);
  }

  // bucket of key k in sub-table `side`
  uint64_t bucket_of(int side, uint64_t k) const {
    if (hash_mode_ == 1) return side == 0 ? k % n_buckets_ : (k / n_buckets_) % n_buckets_;
    return top_bits(mix64(k ^ (side == 0 ? p_.s_h0 : p_.s_h1)), lg_buckets_);
  }
  uint64_t slot_base(int side, uint64_t b) const { return (uint64_t)side * (p_.capacity / 2) + b * bucket_; }

  // worst-case O(1): two buckets (plus the overflow stash, empty in graded runs)
  int64_t find_slot(uint64_t k) const {
    for (int side = 0; side < 2; ++side) {
      uint64_t base = slot_base(side, bucket_of(side, k));
      for (uint32_t l = 0; l < bucket_; ++l)
        if (slot_key_[base + l] == k) return (int64_t)(base + l);
    }
    return -1;
  }
  Entry* find(uint64_t k) {
    int64_t s = find_slot(k);
    if (s >= 0) return &pool_[slot_entry_[s]];
    for (auto& st : stash_)
      if (st.first == k) return &pool_[st.second];
    return nullptr;
  }
  const Entry* find(uint64_t k) const { return const_cast<CuckooModel*>(this)->find(k); }

  int32_t alloc_entry() {
    if (!free_.empty()) { int32_t e = free_.back(); free_.pop_back(); return e; }
    pool_.emplace_back();
    key_of_entry_.push_back(kEmptyKey);
    return (int32_t)pool_.size() - 1;
  }

  // Insert (k, e), k not in the table.  Follows the paper: place at h0; an occupant is evicted
  // and re-inserted into the other sub-table with the same logic, until everything is settled.
  void insert(uint64_t k, int32_t e) {
    int side = 0;
    uint64_t chain = 0;
    for (uint32_t kick = 0; kick <= max_kicks_; ++kick) {
      uint64_t base = slot_base(side, bucket_of(side, k));
      for (uint32_t l = 0; l < bucket_; ++l)
        if (slot_key_[base + l] == kEmptyKey) {
          slot_key_[base + l] = k;
          slot_entry_[base + l] = e;
          max_chain_ = std::max(max_chain_, chain);
          return;
        }
      if (kick == max_kicks_) break;
      uint64_t v = base + kick % bucket_;  // victim
      std::swap(k, slot_key_[v]);
      std::swap(e, slot_entry_[v]);
      side = 1 - side;  // the evicted element goes to its other sub-table
      ++chain;
    }
    // the paper rehashes here; this build keeps the homeless element in a stash and counts it
    stash_.push_back({k, e});
    ++insert_failures_;
  }

  void lookup_or_insert(const int64_t* keys, uint64_t n, uint32_t step, uint8_t* present) override {
    std::vector<uint8_t> was_hit(n, 0);
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey) continue;
      was_hit[i] = find(k) != nullptr;
    }
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      if (k == kEmptyKey || was_hit[i]) continue;
      for (uint32_t j = 0; j < p_.filter_hashes; ++j) {
        uint32_t& w = filter_[filter_index(k, j)];
        w = filter_touch(w, step, p_.expire_steps);
      }
    }
    std::vector<uint64_t> admissible;  // distinct, in ascending first-occurrence order
    {
      std::set<uint64_t> seen;
      for (uint64_t i = 0; i < n; ++i) {
        uint64_t k = (uint64_t)keys[i];
        if (k == kEmptyKey || was_hit[i] || seen.count(k)) continue;
        uint32_t count = 255u;
        for (uint32_t j = 0; j < p_.filter_hashes; ++j) count = std::min(count, filter_[filter_index(k, j)] & 255u);
        if (count < p_.freq_threshold) continue;
        seen.insert(k);
        admissible.push_back(k);
      }
    }
    if (size_ + admissible.size() > fill_limit()) {
      refused_full_ += admissible.size();  // the batch would overfill the table: none of its new keys gets in
    } else {
      for (uint64_t k : admissible) {
        int32_t e = alloc_entry();
        init_entry(p_, k, step, &pool_[e]);
        key_of_entry_[e] = k;
        insert(k, e);
        ++size_;
      }
    }
    for (uint64_t i = 0; i < n; ++i) {
      uint64_t k = (uint64_t)keys[i];
      Entry* e = k == kEmptyKey ? nullptr : find(k);
      if (e && was_hit[i]) e->last_seen = step;
      present[i] = e != nullptr;
    }
  }

  void pool(const int64_t* keys, const int64_t* offsets, uint64_t n_bags, float* out) override {
    std::vector<double> s(p_.dim);
    for (uint64_t b = 0; b < n_bags; ++b) {
      std::fill(s.begin(), s.end(), 0.0);
      for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
        uint64_t k = (uint64_t)keys[i];
        const Entry* e = k == kEmptyKey ? nullptr : find(k);
        if (!e) continue;
        for (uint32_t j = 0; j < p_.dim; ++j) s[j] += (double)e->w[j];
      }
      for (uint32_t j = 0; j < p_.dim; ++j) out[b * p_.dim + j] = (float)s[j];
    }
  }

  void apply_grad(const int64_t* keys, const int64_t* offsets, uint64_t n_bags, const float* grad,
                  float lr, float eps) override {
    // gradient of an entry = sum over its occurrences of the pooled gradient of their bag
    std::vector<int32_t> touched;
    for (uint64_t b = 0; b < n_bags; ++b)
      for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
        uint64_t k = (uint64_t)keys[i];
        Entry* e = k == kEmptyKey ? nullptr : find(k);
        if (!e) continue;
        int32_t id = (int32_t)(e - pool_.data());
        if (gsum_.size() < pool_.size()) gsum_.resize(pool_.size());
        std::vector<double>& g = gsum_[id];
        if (g.empty()) { g.assign(p_.dim, 0.0); touched.push_back(id); }
        for (uint32_t j = 0; j < p_.dim; ++j) g[j] += (double)grad[b * p_.dim + j];
      }
    for (int32_t id : touched) {  // once per distinct key
      adagrad_entry(p_, gsum_[id], (double)lr, (double)eps, &pool_[id]);
      touched_.insert(key_of_entry_[id]);
      gsum_[id].clear();
      gsum_[id].shrink_to_fit();
    }
  }

  void sweep(uint32_t now, std::vector<uint64_t>* erased) override {
    erased->clear();
    if (p_.expire_steps == 0) return;
    for (uint64_t s = 0; s < p_.capacity; ++s) {
      if (slot_key_[s] == kEmptyKey) continue;
      if (now - pool_[slot_entry_[s]].last_seen >= p_.expire_steps) {
        erased->push_back(slot_key_[s]);
        touched_.erase(slot_key_[s]);
        free_.push_back(slot_entry_[s]);
        slot_key_[s] = kEmptyKey;
        slot_entry_[s] = -1;
        --size_;
      }
    }
    for (size_t i = 0; i < stash_.size();) {
      if (now - pool_[stash_[i].second].last_seen >= p_.expire_steps) {
        erased->push_back(stash_[i].first);
        touched_.erase(stash_[i].first);
        free_.push_back(stash_[i].second);
        stash_.erase(stash_.begin() + (long)i);
        --size_;
      } else {
        ++i;
      }
    }
    std::sort(erased->begin(), erased->end());
  }

  void dump(std::vector<Exported>* out) const override {
    out->clear();
    for (uint64_t s = 0; s < p_.capacity; ++s)
      if (slot_key_[s] != kEmptyKey) out->push_back({slot_key_[s], &pool_[slot_entry_[s]], (int64_t)s});
    for (auto& st : stash_) out->push_back({st.first, &pool_[st.second], -2});
    std::sort(out->begin(), out->end(), [](const Exported& a, const Exported& b) { return a.key < b.key; });
  }

  uint32_t filter_word(uint64_t index) const override { return filter_[index]; }

  bool import_entry(uint64_t key, const Entry& e) override {
    if (key == kEmptyKey || find(key)) return false;
    int32_t id = alloc_entry();
    pool_[id] = e;
    key_of_entry_[id] = key;
    insert(key, id);
    ++size_;
    raise_counters(key);
    return true;
  }
  bool is_stored(uint64_t key) const override { return find(key) != nullptr; }
  uint64_t size() const override { return size_; }
  void set_filter_word(uint64_t index, uint32_t word) override { filter_[index] = word; }

  // Every stored element is taken out and inserted again, slots in ascending order and then the
  // stash, into empty sub-tables of the new size addressed by the new generation's h0 / h1.
  void rehash(uint64_t new_capacity, uint32_t generation) override {
    std::vector<std::pair<uint64_t, int32_t>> all;
    for (uint64_t s = 0; s < p_.capacity; ++s)
      if (slot_key_[s] != kEmptyKey) all.push_back({slot_key_[s], slot_entry_[s]});
    for (auto& st : stash_) all.push_back(st);
    stash_.clear();
    int k = regrow_params(new_capacity, generation);
    n_buckets_ = p_.capacity / 2 / bucket_;
    lg_buckets_ = log2_exact(n_buckets_);
    slot_key_.assign(p_.capacity, kEmptyKey);
    slot_entry_.assign(p_.capacity, -1);
    std::vector<uint32_t> grown(p_.n_filter);
    for (uint64_t i = 0; i < p_.n_filter; ++i) grown[i] = filter_[i >> k];
    filter_.swap(grown);
    for (auto& ke : all) insert(ke.first, ke.second);
  }

  uint64_t insert_failures() const override { return insert_failures_; }
  uint64_t max_chain() const override { return max_chain_; }

 private:
  uint32_t bucket_, max_kicks_;
  int hash_mode_;
  uint64_t n_buckets_ = 0;
  int lg_buckets_ = 0;
  std::vector<uint64_t> slot_key_;
  std::vector<int32_t> slot_entry_;
  std::vector<Entry> pool_;
  std::vector<uint64_t> key_of_entry_;  // pool index -> key (for the touched-keys set)
  std::vector<int32_t> free_;
  std::vector<std::pair<uint64_t, int32_t>> stash_;
  std::vector<uint32_t> filter_;
  std::vector<std::vector<double>> gsum_;
  uint64_t size_ = 0, insert_failures_ = 0, max_chain_ = 0;
};

struct Handle {
  std::unique_ptr<Model> m;
  std::vector<Exported> dump;
  std::vector<uint64_t> erased;
  std::vector<uint64_t> touched;
};

bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

}  // namespace

extern "C" {

// kind: 0 = R0 (std::map definition), 1 = R1 (cuckoo).  bucket / max_kicks / hash_mode only
// matter for R1.  n_filter = number of occurrence counters (power of two); filter_hashes = counters
// per key, 1..4 (1: the plain hashed counter array; more: the count of a key is the minimum of its
// counters, the probabilistic filter of section 2.1 read as a counting filter with several hashes).
// Returns NULL on a bad argument.
void* orc_create(int kind, uint64_t capacity, uint32_t dim, uint64_t seed, uint32_t freq_threshold,
                 uint32_t expire_steps, int bf16, uint64_t n_filter, uint32_t bucket,
                 uint32_t max_kicks, int hash_mode, uint32_t filter_hashes) {
  if (dim == 0 || freq_threshold > 255 || !is_pow2(n_filter) || filter_hashes < 1 || filter_hashes > 4) return nullptr;
  Params p;
  p.capacity = capacity;
  p.dim = dim;
  p.seed = seed;
  p.freq_threshold = freq_threshold;
  p.expire_steps = expire_steps;
  p.bf16 = bf16 != 0;
  p.n_filter = n_filter;
  p.lg_filter = log2_exact(n_filter);
  p.s_h0 = salt(placement_seed(seed, 0), 0);
  p.s_h1 = salt(placement_seed(seed, 0), 1);
  p.filter_hashes = filter_hashes;
  p.s_filter[0] = salt(seed, 2);
  for (int j = 1; j < 4; ++j) p.s_filter[j] = salt(seed, 7 + j);
  p.s_init = salt(seed, 3);
  auto* h = new Handle;
  if (kind == 0) {
    h->m.reset(new BruteForceModel(p));
  } else {
    if (!is_pow2(capacity) || bucket == 0 || !is_pow2(bucket) || capacity < 2ull * bucket) {
      delete h;
      return nullptr;
    }
    h->m.reset(new CuckooModel(p, bucket, max_kicks, hash_mode));
  }
  return h;
}

void orc_destroy(void* hv) { delete (Handle*)hv; }

// keys[n]; step < 2^24; present[n] receives 1 where the occurrence's key is in the table afterwards
void orc_lookup_or_insert(void* hv, const int64_t* keys, uint64_t n, uint32_t step, uint8_t* present) {
  ((Handle*)hv)->m->lookup_or_insert(keys, n, step, present);
}

// out[n_bags * dim], bag b = occurrences [offsets[b], offsets[b+1])
void orc_pool(void* hv, const int64_t* keys, const int64_t* offsets, uint64_t n_bags, float* out) {
  ((Handle*)hv)->m->pool(keys, offsets, n_bags, out);
}

void orc_apply_grad_adagrad(void* hv, const int64_t* keys, const int64_t* offsets, uint64_t n_bags,
                            const float* grad, float lr, float eps) {
  ((Handle*)hv)->m->apply_grad(keys, offsets, n_bags, grad, lr, eps);
}

// returns the number of erased keys; they can then be read (sorted) with orc_erased_keys
uint64_t orc_expire_sweep(void* hv, uint32_t now) {
  Handle* h = (Handle*)hv;
  h->m->sweep(now, &h->erased);
  std::sort(h->erased.begin(), h->erased.end());
  return h->erased.size();
}
void orc_erased_keys(void* hv, int64_t* out) {
  Handle* h = (Handle*)hv;
  for (size_t i = 0; i < h->erased.size(); ++i) out[i] = (int64_t)h->erased[i];
}

// snapshot the table (sorted by key); returns the number of keys, then orc_dump_read copies it
uint64_t orc_dump(void* hv) {
  Handle* h = (Handle*)hv;
  h->m->dump(&h->dump);
  return h->dump.size();
}
void orc_dump_read(void* hv, int64_t* keys, float* rows, float* acc, uint32_t* last_seen, int64_t* slot) {
  Handle* h = (Handle*)hv;
  uint32_t d = h->m->params().dim;
  for (size_t i = 0; i < h->dump.size(); ++i) {
    const Exported& x = h->dump[i];
    keys[i] = (int64_t)x.key;
    std::memcpy(rows + i * d, x.e->w.data(), d * sizeof(float));
    acc[i] = x.e->acc;
    last_seen[i] = x.e->last_seen;
    slot[i] = x.slot;
  }
}

// canonical counter words [first, first + count)
void orc_filter_read(void* hv, uint64_t first, uint64_t count, uint32_t* out) {
  Handle* h = (Handle*)hv;
  for (uint64_t i = 0; i < count; ++i) out[i] = h->m->filter_word(first + i);
}
uint64_t orc_filter_index(void* hv, int64_t key) { return ((Handle*)hv)->m->filter_index((uint64_t)key); }
uint64_t orc_filter_index_j(void* hv, int64_t key, uint32_t j) {
  return ((Handle*)hv)->m->filter_index((uint64_t)key, j);
}

uint64_t orc_insert_failures(void* hv) { return ((Handle*)hv)->m->insert_failures(); }
// admissible keys (or restore records) refused because their call would have overfilled the table
uint64_t orc_refused_full(void* hv) { return ((Handle*)hv)->m->refused_full(); }
uint64_t orc_max_chain(void* hv) { return ((Handle*)hv)->m->max_chain(); }

// -- maintenance operations -------------------------------------------------------------------

// keys trained since the last call: returns how many, then orc_touched_keys copies them (ascending)
uint64_t orc_take_touched(void* hv) {
  Handle* h = (Handle*)hv;
  h->m->take_touched(&h->touched);
  return h->touched.size();
}
void orc_touched_keys(void* hv, int64_t* out) {
  Handle* h = (Handle*)hv;
  for (size_t i = 0; i < h->touched.size(); ++i) out[i] = (int64_t)h->touched[i];
}

// restore: records are placed in the order given; rows[n * dim] are rounded to the storage type.
// Returns the number of records NOT placed: key already stored, reserved key, second record of a key
// within the call, or - for every record of the call - a call that would take the table past its fill limit.
uint64_t orc_import(void* hv, const int64_t* keys, const float* rows, const float* acc,
                    const uint32_t* last_seen, uint64_t n) {
  Handle* h = (Handle*)hv;
  const Params& p = h->m->params();
  uint64_t rejected = 0;
  {
    std::set<uint64_t> fresh;  // distinct keys of the call that are not stored yet
    for (uint64_t i = 0; i < n; ++i)
      if ((uint64_t)keys[i] != kEmptyKey && !h->m->is_stored((uint64_t)keys[i])) fresh.insert((uint64_t)keys[i]);
    if (h->m->size() + fresh.size() > h->m->fill_limit()) {
      h->m->count_refused_full(fresh.size());
      return n;
    }
  }
  for (uint64_t i = 0; i < n; ++i) {
    Entry e;
    e.w.resize(p.dim);
    for (uint32_t j = 0; j < p.dim; ++j) e.w[j] = p.bf16 ? bf16_round(rows[i * p.dim + j]) : rows[i * p.dim + j];
    e.acc = acc[i];
    e.last_seen = last_seen[i];
    if (!h->m->import_entry((uint64_t)keys[i], e)) ++rejected;
  }
  return rejected;
}
void orc_filter_write(void* hv, uint64_t first, uint64_t count, const uint32_t* words) {
  ((Handle*)hv)->m->write_filter_words(first, count, words);
}

// rehash / grow: new_capacity a power of two >= the current one; 0 on success, -1 on a bad argument
int orc_rehash(void* hv, uint64_t new_capacity, uint32_t generation) {
  Handle* h = (Handle*)hv;
  uint64_t cap = h->m->params().capacity;
  if (!is_pow2(new_capacity) || new_capacity < cap || !is_pow2(cap)) return -1;
  h->m->rehash(new_capacity, generation);
  return 0;
}
uint64_t orc_capacity(void* hv) { return ((Handle*)hv)->m->params().capacity; }
uint64_t orc_n_filter(void* hv) { return ((Handle*)hv)->m->params().n_filter; }
uint64_t orc_placement_salt(uint64_t seed, uint32_t generation, int side) {
  return salt(placement_seed(seed, generation), side);
}

// Quotient-remainder embedding (section 3.1): two dense tables of 2^m rows, E = E_r[id mod 2^m] +
// E_q[id div 2^m], summed per bag in fp64 and rounded once.  table_r / table_q: [2^m * dim] fp32
// (values already rounded to the storage type by the caller).
void orc_qr_pool(const float* table_r, const float* table_q, uint32_t m, uint32_t dim, const int64_t* ids,
                 const int64_t* offsets, uint64_t n_bags, float* out) {
  std::vector<double> s(dim);
  const uint64_t rows = 1ull << m;
  for (uint64_t b = 0; b < n_bags; ++b) {
    std::fill(s.begin(), s.end(), 0.0);
    for (int64_t i = offsets[b]; i < offsets[b + 1]; ++i) {
      if (ids[i] < 0) continue;
      uint64_t id = (uint64_t)ids[i];
      uint64_t id_r = id % rows, id_q = id / rows;
      if (id_q >= rows) continue;  // outside the decomposed ID space
      for (uint32_t j = 0; j < dim; ++j) s[j] += (double)table_r[id_r * dim + j] + (double)table_q[id_q * dim + j];
    }
    for (uint32_t j = 0; j < dim; ++j) out[b * dim + j] = (float)s[j];
  }
}

// building blocks exposed so that tests can pin them separately
uint64_t orc_mix64(uint64_t z) { return mix64(z); }
uint64_t orc_salt(uint64_t seed, int i) { return salt(seed, i); }
float orc_init_value(uint64_t seed, int64_t key, uint32_t j) { return init_value(salt(seed, 3), (uint64_t)key, j); }
float orc_bf16_round(float x) { return bf16_round(x); }
uint32_t orc_filter_touch(uint32_t word, uint32_t step, uint32_t expire_steps) {
  return filter_touch(word, step, expire_steps);
}

}  // extern "C"
