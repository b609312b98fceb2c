// CPU oracle for the embedding hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, single-threaded statement of what the path computes, written from
// the paper's definitions so that it can be checked against them by eye.  Only the
// tests, the smoke check and the benchmark's cpu_baseline leg may load it; the HIP
// library shares no code with it and never calls it.
//
// What it computes, and where the paper defines it:
//   hash      ID -> row of the slot's table.  The paper only says a global hashing
//             function locates the storage of a parameter (section 4.2.2, "Persia
//             Memory Management"); the function itself is this build's choice and is
//             written out below (mix64).
//   lookup    lookup_{w_emb}(x^ID): the embedding vectors that correspond to the IDs
//             of a sample, one group per ID-type feature ("slot"), concatenated over
//             slots (section 2.1).  Inside a slot the vectors are aggregated by a sum
//             (the "potential aggregation" of step 4 in section 4.1), duplicates
//             counted with their multiplicity.
//   dedup     the lossless index form of a batch (section 4.2.3, "Lossless
//             compression"): unique key -> the list of sample positions that hold it.
//             Keys here are (table,row) after hashing, ascending; positions are bag
//             indices b*S+s in batch order.
//   gradient  F'^emb: gradient of the loss w.r.t. each touched row given the gradient
//             w.r.t. the pooled activations (step 7 in section 4.1).  For sum pooling
//             this is the sum of the upstream gradients of every bag occurrence.
//   update    w^emb_{t+1} = w^emb_t - Omega^emb(F'^emb) (Algorithm 1, backward task;
//             equation (2)), once per unique row per batch, with the optimizer state
//             stored beside the row (section 4.2.2).  Omega^emb is SGD or row-wise
//             Adagrad (one fp32 accumulator per row, fed by the mean over the row of
//             the squared gradient, eps outside the square root).
//
// All floating-point accumulation is fp64; each stored quantity is rounded once, from the
// fp64 result straight to its storage type (fp32, or bf16 for bf16 tables: never fp64 -> fp32 -> bf16,
// whose two roundings can differ from one at a bf16 tie).
// Parity pins live in tests/test_oracle_*.py.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <unordered_map>
#include <vector>

namespace {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { OPT_SGD = 0, OPT_ROWWISE_ADAGRAD = 1 };
enum { HASH_IDENTITY_MOD = 0, HASH_MIX_MOD = 1 };

// 64-bit bijective mixer: xor-shift 31, multiply, xor-shift 29, multiply, xor-shift 32.
uint64_t mix64(uint64_t z) {
  z ^= z >> 31;
  z *= 0x9FB21C651E98DF25ull;
  z ^= z >> 29;
  z *= 0xC2B2AE3D27D4EB4Full;
  z ^= z >> 32;
  return z;
}

// fp32 -> bf16 (round to nearest, ties to even; NaN kept quiet) -> fp32.
float round_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0) {
    u = (u | 0x00400000u) & 0xFFFF0000u;  // quiet NaN, payload truncated
  } else {
    uint32_t lower = u & 0xFFFFu;
    uint32_t upper = u & 0xFFFF0000u;
    bool odd = (u >> 16) & 1u;
    if (lower > 0x8000u || (lower == 0x8000u && odd)) upper += 0x10000u;
    u = upper;
  }
  float r;
  std::memcpy(&r, &u, 4);
  return r;
}

// fp64 -> bf16 in ONE rounding (nearest, ties to even), returned widened to fp32.  A bf16 value is
// m * 2^(e-7) with an 8-bit integer m (7 stored bits + the leading one) and the exponent range of
// fp32; below 2^-126 the spacing stays 2^-133 (subnormals).  So: find the spacing for |v|'s binade,
// divide (exact: a power of two), round the quotient to the nearest integer, ties to even, multiply
// back (exact).  Beyond the largest finite bf16 the result is infinity.
float round_bf16_once(double v) {
  if (std::isnan(v)) return std::numeric_limits<float>::quiet_NaN();
  if (std::isinf(v) || v == 0.0) return (float)v;
  int e;
  std::frexp(v, &e);           // |v| = f * 2^e with f in [0.5, 1): the binade is [2^(e-1), 2^e)
  int q = e - 1 - 7;           // spacing 2^q of bf16 values in that binade
  if (q < -133) q = -133;      // subnormal range
  const double scaled = std::ldexp(v, -q);
  const double r = std::nearbyint(scaled);   // the default rounding mode: to nearest, ties to even
  const double out = std::ldexp(r, q);
  const double max_bf16 = std::ldexp(255.0, 127 - 7);  // 0x7F7F: (2 - 2^-7) * 2^127
  if (std::fabs(out) > max_bf16) return std::copysign(std::numeric_limits<float>::infinity(), (float)v);
  return (float)out;           // exact: every finite bf16 value is an fp32 value
}

// Initial value of element d of row r of table t: 24 random bits k from a counter
// hash, mapped to lo + (hi-lo)*(k/2^24) as (k - 2^23)*scale + mid with one fp32
// multiply and one fp32 add (no fused multiply-add).
float init_value(uint64_t seed, uint32_t t, uint64_t r, uint32_t dim, uint32_t d, float lo, float hi) {
  uint64_t table_key = mix64(seed + (uint64_t)(t + 1) * 0x9E3779B97F4A7C15ull);
  uint64_t h = mix64(table_key + r * (uint64_t)dim + d);
  int32_t k = (int32_t)(h >> 40) - (1 << 23);
  volatile float scale = (hi - lo) * 5.9604644775390625e-08f;  // 2^-24
  volatile float mid = (hi + lo) * 0.5f;
  volatile float prod = (float)k * scale;
  volatile float v = prod + mid;
  return v;
}

struct Table {
  uint64_t rows = 0;
  uint32_t dim = 0;
  int dtype = DT_F32;
  bool dense = false;
  std::vector<float> w;    // dense: rows*dim; sparse: touched rows, in order of first touch
  std::vector<float> acc;  // one per stored row
  std::unordered_map<uint64_t, size_t> where;  // sparse: row -> index of its storage
};

struct Oracle {
  std::vector<Table> tables;
  std::vector<uint32_t> slot_table;
  std::vector<uint64_t> slot_salt;
  std::vector<uint32_t> slot_col;
  uint32_t width = 0;
  int hash_kind = HASH_MIX_MOD, opt = OPT_SGD;
  float lr = 0, eps = 0, acc_init = 0, init_lo = 0, init_hi = 0;
  uint64_t init_seed = 0;
  // results of the last dedup / backward
  std::vector<uint64_t> unique_keys;
  std::vector<uint32_t> seg_off;
  std::vector<uint32_t> seg_bags;
  std::vector<double> grad;  // ragged: dim(table(u)) doubles per unique key u
};

float store_round(const Table& t, double v) { return t.dtype == DT_BF16 ? round_bf16_once(v) : (float)v; }

void init_row(const Oracle& o, uint32_t ti, const Table& t, uint64_t r, float* dst) {
  for (uint32_t d = 0; d < t.dim; ++d) {
    float v = init_value(o.init_seed, ti, r, t.dim, d, o.init_lo, o.init_hi);
    dst[d] = t.dtype == DT_BF16 ? round_bf16(v) : v;
  }
}

// Index of row r's storage (sparse mode materialises the row from its initial value on first touch).
size_t row_index(Oracle& o, uint32_t ti, uint64_t r) {
  Table& t = o.tables[ti];
  if (t.dense) return (size_t)r;
  auto it = t.where.find(r);
  if (it != t.where.end()) return it->second;
  size_t idx = t.acc.size();
  t.w.resize((idx + 1) * (size_t)t.dim);
  init_row(o, ti, t, r, &t.w[idx * (size_t)t.dim]);
  t.acc.push_back(o.acc_init);
  t.where.emplace(r, idx);
  return idx;
}

uint64_t hash_row(const Oracle& o, uint64_t id, uint32_t slot) {
  const Table& t = o.tables[o.slot_table[slot]];
  if (o.hash_kind == HASH_IDENTITY_MOD) return id % t.rows;
  return mix64(id + o.slot_salt[slot]) % t.rows;
}

}  // namespace

extern "C" {

uint64_t orc_mix64(uint64_t z) { return mix64(z); }
float orc_round_bf16(float x) { return round_bf16(x); }
float orc_round_bf16_once(double v) { return round_bf16_once(v); }
float orc_init_value(uint64_t seed, uint32_t t, uint64_t r, uint32_t dim, uint32_t d, float lo, float hi) {
  return init_value(seed, t, r, dim, d, lo, hi);
}

void* orc_create(uint32_t num_tables, const uint64_t* rows, const uint32_t* dims, const int32_t* dtypes,
                 uint32_t num_slots, const uint32_t* slot_table, const uint64_t* slot_salt, int hash_kind, int opt,
                 float lr, float eps, float acc_init, uint64_t init_seed, float init_lo, float init_hi,
                 int dense) {
  Oracle* o = new Oracle();
  o->hash_kind = hash_kind;
  o->opt = opt;
  o->lr = lr;
  o->eps = eps;
  o->acc_init = acc_init;
  o->init_seed = init_seed;
  o->init_lo = init_lo;
  o->init_hi = init_hi;
  o->tables.resize(num_tables);
  for (uint32_t i = 0; i < num_tables; ++i) {
    Table& t = o->tables[i];
    t.rows = rows[i];
    t.dim = dims[i];
    t.dtype = dtypes[i];
    t.dense = dense != 0;
    if (t.dense) {
      t.w.resize((size_t)t.rows * t.dim);
      t.acc.assign((size_t)t.rows, acc_init);
      for (uint64_t r = 0; r < t.rows; ++r) init_row(*o, i, t, r, &t.w[(size_t)r * t.dim]);
    }
  }
  uint32_t col = 0;
  for (uint32_t s = 0; s < num_slots; ++s) {
    if (slot_table[s] >= num_tables) { delete o; return nullptr; }
    o->slot_table.push_back(slot_table[s]);
    o->slot_salt.push_back(slot_salt[s]);
    o->slot_col.push_back(col);
    col += o->tables[slot_table[s]].dim;
  }
  o->width = col;
  return o;
}

void orc_destroy(void* h) { delete (Oracle*)h; }

uint32_t orc_pooled_width(void* h) { return ((Oracle*)h)->width; }

// Rows of the sparse tables that have been touched so far (dense tables: all rows).
uint64_t orc_rows_stored(void* h, uint32_t table) { return ((Oracle*)h)->tables[table].acc.size(); }

// hash: rows_out[i] = row of id i in the table of its slot; slot of a bag = bag mod S.
int orc_hash_rows(void* h, const uint64_t* ids, const int32_t* offsets, uint32_t B, uint32_t* rows_out) {
  Oracle& o = *(Oracle*)h;
  uint32_t S = (uint32_t)o.slot_table.size();
  for (uint64_t bag = 0; bag < (uint64_t)B * S; ++bag)
    for (int32_t i = offsets[bag]; i < offsets[bag + 1]; ++i)
      rows_out[i] = (uint32_t)hash_row(o, ids[i], (uint32_t)(bag % S));
  return 0;
}

// lookup + per-slot sum pooling: pooled[b, col(s) + d] = sum over the bag's ids of W[row][d].
int orc_lookup_pool(void* h, const uint64_t* ids, const int32_t* offsets, uint32_t B, float* pooled) {
  Oracle& o = *(Oracle*)h;
  uint32_t S = (uint32_t)o.slot_table.size();
  std::vector<double> sum;
  for (uint32_t b = 0; b < B; ++b) {
    for (uint32_t s = 0; s < S; ++s) {
      uint64_t bag = (uint64_t)b * S + s;
      uint32_t ti = o.slot_table[s];
      uint32_t D = o.tables[ti].dim;
      sum.assign(D, 0.0);
      for (int32_t i = offsets[bag]; i < offsets[bag + 1]; ++i) {
        size_t idx = row_index(o, ti, hash_row(o, ids[i], s));
        const float* w = &o.tables[ti].w[idx * (size_t)D];
        for (uint32_t d = 0; d < D; ++d) sum[d] += (double)w[d];
      }
      float* out = pooled + (size_t)b * o.width + o.slot_col[s];
      for (uint32_t d = 0; d < D; ++d) out[d] = (float)sum[d];
    }
  }
  return 0;
}

// dedup: every occurrence becomes (key = table<<32 | row, bag); a stable sort by key groups
// them, keeping batch order inside a group.
int orc_dedup(void* h, const uint64_t* ids, const int32_t* offsets, uint32_t B) {
  Oracle& o = *(Oracle*)h;
  uint32_t S = (uint32_t)o.slot_table.size();
  std::vector<std::pair<uint64_t, uint32_t>> occ;
  occ.reserve((size_t)offsets[(size_t)B * S]);
  for (uint64_t bag = 0; bag < (uint64_t)B * S; ++bag) {
    uint32_t s = (uint32_t)(bag % S);
    for (int32_t i = offsets[bag]; i < offsets[bag + 1]; ++i)
      occ.emplace_back(((uint64_t)o.slot_table[s] << 32) | hash_row(o, ids[i], s), (uint32_t)bag);
  }
  std::stable_sort(occ.begin(), occ.end(),
                   [](const std::pair<uint64_t, uint32_t>& a, const std::pair<uint64_t, uint32_t>& b) {
                     return a.first < b.first;
                   });
  o.unique_keys.clear();
  o.seg_off.clear();
  o.seg_bags.resize(occ.size());
  for (size_t i = 0; i < occ.size(); ++i) {
    if (i == 0 || occ[i].first != occ[i - 1].first) {
      o.unique_keys.push_back(occ[i].first);
      o.seg_off.push_back((uint32_t)i);
    }
    o.seg_bags[i] = occ[i].second;
  }
  o.seg_off.push_back((uint32_t)occ.size());
  return 0;
}

void orc_dedup_sizes(void* h, uint64_t* U, uint64_t* N) {
  Oracle& o = *(Oracle*)h;
  *U = o.unique_keys.size();
  *N = o.seg_bags.size();
}

void orc_dedup_copy(void* h, uint64_t* unique_keys, uint32_t* seg_off, uint32_t* seg_bags) {
  Oracle& o = *(Oracle*)h;
  std::copy(o.unique_keys.begin(), o.unique_keys.end(), unique_keys);
  std::copy(o.seg_off.begin(), o.seg_off.end(), seg_off);
  std::copy(o.seg_bags.begin(), o.seg_bags.end(), seg_bags);
}

// gradient per unique row from the last dedup: G[u][d] = sum over the row's bags of
// d_pooled[b, col(s) + d], one term per occurrence.
int orc_gradient(void* h, uint32_t B, const float* d_pooled) {
  Oracle& o = *(Oracle*)h;
  uint32_t S = (uint32_t)o.slot_table.size();
  (void)B;
  o.grad.clear();
  for (size_t u = 0; u < o.unique_keys.size(); ++u) {
    uint32_t ti = (uint32_t)(o.unique_keys[u] >> 32);
    uint32_t D = o.tables[ti].dim;
    size_t base = o.grad.size();
    o.grad.resize(base + D, 0.0);
    for (uint32_t j = o.seg_off[u]; j < o.seg_off[u + 1]; ++j) {
      uint32_t bag = o.seg_bags[j];
      const float* g = d_pooled + (size_t)(bag / S) * o.width + o.slot_col[bag % S];
      for (uint32_t d = 0; d < D; ++d) o.grad[base + d] += (double)g[d];
    }
  }
  return 0;
}

uint64_t orc_grad_size(void* h) { return ((Oracle*)h)->grad.size(); }
void orc_grad_copy(void* h, double* out) {
  Oracle& o = *(Oracle*)h;
  std::copy(o.grad.begin(), o.grad.end(), out);
}

// optimizer: one application per unique row, using the gradient of the last orc_gradient.
int orc_apply_update(void* h) {
  Oracle& o = *(Oracle*)h;
  size_t base = 0;
  for (size_t u = 0; u < o.unique_keys.size(); ++u) {
    uint32_t ti = (uint32_t)(o.unique_keys[u] >> 32);
    uint64_t r = o.unique_keys[u] & 0xFFFFFFFFull;
    Table& t = o.tables[ti];
    uint32_t D = t.dim;
    size_t idx = row_index(o, ti, r);
    float* w = &t.w[idx * (size_t)D];
    const double* G = &o.grad[base];
    if (o.opt == OPT_SGD) {
      for (uint32_t d = 0; d < D; ++d) w[d] = store_round(t, (double)w[d] - (double)o.lr * G[d]);
    } else {
      double sq = 0.0;
      for (uint32_t d = 0; d < D; ++d) sq += G[d] * G[d];
      double a = (double)t.acc[idx] + sq / (double)D;
      double denom = std::sqrt(a) + (double)o.eps;
      for (uint32_t d = 0; d < D; ++d) w[d] = store_round(t, (double)w[d] - (double)o.lr * G[d] / denom);
      t.acc[idx] = (float)a;
    }
    base += D;
  }
  return 0;
}

// backward of one batch: dedup, gradient per unique row, optimizer update.
int orc_backward_update(void* h, const uint64_t* ids, const int32_t* offsets, uint32_t B, const float* d_pooled) {
  orc_dedup(h, ids, offsets, B);
  orc_gradient(h, B, d_pooled);
  return orc_apply_update(h);
}

int orc_read_rows(void* h, uint32_t table, const uint64_t* rows, uint64_t n, float* w_out, float* acc_out) {
  Oracle& o = *(Oracle*)h;
  if (table >= o.tables.size()) return -1;
  Table& t = o.tables[table];
  for (uint64_t i = 0; i < n; ++i) {
    if (rows[i] >= t.rows) return -1;
    size_t idx = row_index(o, table, rows[i]);
    if (w_out) std::copy(&t.w[idx * (size_t)t.dim], &t.w[(idx + 1) * (size_t)t.dim], w_out + i * (size_t)t.dim);
    if (acc_out) acc_out[i] = t.acc[idx];
  }
  return 0;
}

// Overwrites rows (values are rounded to the table's storage type); acc may be null.
int orc_write_rows(void* h, uint32_t table, const uint64_t* rows, uint64_t n, const float* w_in, const float* acc_in) {
  Oracle& o = *(Oracle*)h;
  if (table >= o.tables.size()) return -1;
  Table& t = o.tables[table];
  for (uint64_t i = 0; i < n; ++i) {
    if (rows[i] >= t.rows) return -1;
    size_t idx = row_index(o, table, rows[i]);
    for (uint32_t d = 0; d < t.dim; ++d) t.w[idx * (size_t)t.dim + d] = store_round(t, (double)w_in[i * (size_t)t.dim + d]);
    if (acc_in) t.acc[idx] = acc_in[i];
  }
  return 0;
}

}  // extern "C"
