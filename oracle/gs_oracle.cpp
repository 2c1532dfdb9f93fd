// Reference ("oracle") implementation of the walk + skip-gram hot path.
//
// THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded CPU
// program whose only job is to say what the right answer is.  Nothing in the
// product path may call it, and it shares no source with the HIP library:
// the Philox generator, the alias sampler and every formula below are written
// out here a second time on purpose.
//
// What is computed follows GraphScale (arXiv 2407.15452):
//   * §2.2 "Node embedding training": random walks from every node, then the
//     skip-gram model with negative sampling on the walks (DeepWalk), with the
//     biased second-order walk of node2vec as the extension.
//   * §3.1: a trainer holds the whole graph topology locally (here: CSR).
//   * §3.2: one iteration touches only the n rows named by the batch (source
//     nodes plus their positively and negatively sampled nodes); the loss is
//     computed on those rows and only those rows are written back.
//   * §3.2 "Synchronization": a barrier follows the write of an iteration, so
//     every read of an iteration sees the values from before that iteration.
// The paper fixes no formula, constant or random-number convention; the
// conventions used here are the ones listed in the design notes of this
// repository and are repeated in the comment of each function.
//
// Floating point: every sampling decision is a single IEEE operation on
// exactly representable inputs; the SGNS arithmetic is done in fp64 and rounded
// once per written element.  Build with -ffp-contract=off.
//
// Parity pins: every function here is pinned by tests/test_oracle_*.py
// (known-answer vectors, closed forms, brute force, library routines).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <deque>
#include <unordered_map>
#include <vector>

extern "C" {

typedef struct {
  int64_t num_nodes;
  int64_t num_entries;
  const void* offsets;  // int32 or int64, num_nodes + 1 entries
  int32_t offset_bits;  // 32 or 64
  const int32_t* nbrs;  // num_entries, each row ascending
  const float* weights; // may be null
} oracle_csr;

typedef struct {
  const float* prob;    // null => uniform
  const int32_t* alias; // segment-local index
} oracle_alias;

enum { ORACLE_OK = 0, ORACLE_EINVAL = -1, ORACLE_EOVERFLOW = -3 };
enum { ORACLE_SYMMETRIZE = 1, ORACLE_DROP_SELF_LOOPS = 2, ORACLE_DEDUPE = 4 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

}  // extern "C"

namespace {

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  Ten rounds; the key is bumped by the Weyl constants
// before every round except the first.
// ---------------------------------------------------------------------------
struct Block4 { uint32_t x[4]; };

Block4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                     uint32_t k0, uint32_t k1) {
  const uint64_t MUL_A = 0xD2511F53ull;  // multiplies word 0
  const uint64_t MUL_B = 0xCD9E8D57ull;  // multiplies word 2
  for (int round = 0; round < 10; ++round) {
    if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    uint64_t pa = MUL_A * c0;
    uint64_t pb = MUL_B * c2;
    uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)pb;
    uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)pa;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  return Block4{{c0, c1, c2, c3}};
}

Block4 philox_keyed(uint64_t seed, uint64_t index, uint32_t c2, uint32_t c3) {
  return philox4x32_10((uint32_t)index, (uint32_t)(index >> 32), c2, c3,
                       (uint32_t)seed, (uint32_t)(seed >> 32));
}

// slot in [0, n): high 64 bits of the 128-bit product r * n.
uint64_t slot_of(uint64_t r, uint64_t n) {
  return (uint64_t)(((unsigned __int128)r * (unsigned __int128)n) >> 64);
}

// 24 random bits as a float in [0, 1): exact in fp32.
float unit_float(uint32_t x) { return (float)(x >> 8) * 0x1p-24f; }

int64_t offset_at(const void* offsets, int32_t bits, int64_t i) {
  return bits == 64 ? ((const int64_t*)offsets)[i]
                    : (int64_t)((const int32_t*)offsets)[i];
}

// One neighbour draw from the row of `cur`, using random block `b`:
// words 0,1 choose the slot; word 2 decides the alias acceptance.
// Returns the position inside the row (0 <= result < deg).
int64_t draw_in_row(const oracle_alias* a, int64_t row_begin, int64_t deg,
                    const Block4& b) {
  uint64_t r = ((uint64_t)b.x[0] << 32) | (uint64_t)b.x[1];
  int64_t j = (int64_t)slot_of(r, (uint64_t)deg);
  if (a != nullptr && a->prob != nullptr) {
    float accept = unit_float(b.x[2]);
    if (!(accept < a->prob[row_begin + j])) j = (int64_t)a->alias[row_begin + j];
  }
  return j;
}

bool row_contains(const oracle_csr* g, int64_t node, int32_t x) {
  int64_t lo = offset_at(g->offsets, g->offset_bits, node);
  int64_t hi = offset_at(g->offsets, g->offset_bits, node + 1);
  return std::binary_search(g->nbrs + lo, g->nbrs + hi, x);
}

float bf16_to_float(uint16_t h) {
  uint32_t bits = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &bits, 4);
  return f;
}

// round-to-nearest-even fp32 -> bf16 (finite inputs only)
uint16_t float_to_bf16(float f) {
  uint32_t bits;
  std::memcpy(&bits, &f, 4);
  uint32_t lsb = (bits >> 16) & 1u;
  bits += 0x7FFFu + lsb;
  return (uint16_t)(bits >> 16);
}

// IEEE binary16 (1 sign, 5 exponent, 10 fraction bits), widened exactly
float f16_to_float(uint16_t h) {
  const int sign = (h >> 15) & 1, ex = (h >> 10) & 31, frac = h & 1023;
  double v;
  if (ex == 0) v = std::ldexp((double)frac, -24);                       // subnormal
  else if (ex == 31) v = frac ? std::nan("") : INFINITY;
  else v = std::ldexp(1.0 + (double)frac / 1024.0, ex - 15);
  return (float)(sign ? -v : v);
}

// fp32 -> binary16, round to nearest even (overflow to infinity)
uint16_t float_to_f16(float f) {
  const uint16_t sign = std::signbit(f) ? 0x8000u : 0u;
  const double a = std::fabs((double)f);
  if (std::isnan(f)) return (uint16_t)(sign | 0x7e00u);
  if (a == 0.0) return sign;
  if (std::isinf(f)) return (uint16_t)(sign | 0x7c00u);
  int ex;
  std::frexp(a, &ex);                          // a = m * 2^ex, m in [0.5, 1)
  int e = ex - 1;                              // a = 1.xxx * 2^e
  if (e < -14) {                               // subnormal range: units of 2^-24
    const double q = std::nearbyint(std::ldexp(a, 24));
    return (uint16_t)(sign | (uint16_t)q);     // q == 1024 is the smallest normal number
  }
  double q = std::nearbyint(std::ldexp(a, 10 - e));   // in [1024, 2048]
  if (q == 2048.0) { q = 1024.0; ++e; }
  if (e > 15) return (uint16_t)(sign | 0x7c00u);
  return (uint16_t)(sign | ((uint16_t)(e + 15) << 10) | (uint16_t)(q - 1024.0));
}

double softplus(double z) {  // log(1 + exp(z)), stable for both signs
  return std::max(z, 0.0) + std::log1p(std::exp(-std::fabs(z)));
}

double sigmoid(double z) {
  if (z >= 0.0) return 1.0 / (1.0 + std::exp(-z));
  double e = std::exp(z);
  return e / (1.0 + e);
}

double read_elem(const void* table, int32_t dtype, int32_t dim, int64_t row, int32_t e) {
  if (dtype == ORACLE_F32) return (double)((const float*)table)[row * dim + e];
  if (dtype == ORACLE_F16) return (double)f16_to_float(((const uint16_t*)table)[row * dim + e]);
  return (double)bf16_to_float(((const uint16_t*)table)[row * dim + e]);
}

void write_elem(void* table, int32_t dtype, int32_t dim, int64_t row, int32_t e, double value) {
  if (dtype == ORACLE_F32) ((float*)table)[row * dim + e] = (float)value;
  else if (dtype == ORACLE_F16) ((uint16_t*)table)[row * dim + e] = float_to_f16((float)value);
  else ((uint16_t*)table)[row * dim + e] = float_to_bf16((float)value);
}

typedef std::unordered_map<int32_t, std::vector<double>> RowSums;

// Gradient of the batch's summed SGNS loss with respect to the rows it names,
// at the given tables, in fp64: d_in[c] = sum_j g_j v_j, d_out[row_j] = g_j u.
int32_t sgns_gradients(const void* w_in, const void* w_out, int64_t num_nodes, int32_t dim,
                       int32_t dtype, const int32_t* centers, const int32_t* contexts,
                       const int32_t* negs, int64_t num_pairs, int32_t k, RowSums& d_in,
                       RowSums& d_out, double* loss_sum_out) {
  auto slot = [&](RowSums& m, int32_t row) -> std::vector<double>& {
    auto it = m.find(row);
    if (it == m.end()) it = m.emplace(row, std::vector<double>((size_t)dim, 0.0)).first;
    return it->second;
  };
  double loss = 0.0;
  std::vector<double> u((size_t)dim), v((size_t)dim);
  for (int64_t i = 0; i < num_pairs; ++i) {
    int32_t c = centers[i];
    if (c < 0 || c >= num_nodes) return ORACLE_EINVAL;
    for (int32_t e = 0; e < dim; ++e) u[(size_t)e] = read_elem(w_in, dtype, dim, c, e);
    std::vector<double>& du = slot(d_in, c);
    for (int32_t j = 0; j <= k; ++j) {
      int32_t row = (j == 0) ? contexts[i] : negs[i * (int64_t)k + (j - 1)];
      if (row < 0 || row >= num_nodes) return ORACLE_EINVAL;
      double x = 0.0;
      for (int32_t e = 0; e < dim; ++e) {
        v[(size_t)e] = read_elem(w_out, dtype, dim, row, e);
        x += u[(size_t)e] * v[(size_t)e];
      }
      double gj;
      if (j == 0) { loss += softplus(-x); gj = sigmoid(x) - 1.0; }
      else        { loss += softplus(x);  gj = sigmoid(x); }
      std::vector<double>& dv = slot(d_out, row);
      for (int32_t e = 0; e < dim; ++e) {
        du[(size_t)e] += gj * v[(size_t)e];
        dv[(size_t)e] += gj * u[(size_t)e];
      }
    }
  }
  *loss_sum_out = loss;
  return ORACLE_OK;
}

}  // namespace

extern "C" {

// Exposed so the tests can check the generator against published
// known-answer vectors.
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  Block4 b = philox4x32_10(ctr[0], ctr[1], ctr[2], ctr[3], key[0], key[1]);
  for (int i = 0; i < 4; ++i) out[i] = b.x[i];
}

// ---------------------------------------------------------------------------
// Topology (§3.1: the trainer keeps the entire graph topology).
// Edge list -> CSR.  Edges with an endpoint outside [0, num_nodes) are dropped.
// Optional: drop self loops, add the reverse of every edge, remove duplicate
// (src, dst) entries keeping the one that came from the lowest input index
// (its weight is the one kept).  Each row is sorted ascending by neighbour id;
// equal neighbours (only without DEDUPE) stay in input order.
// Capacity of nbrs_out / w_out: m entries, 2m with SYMMETRIZE.
// ---------------------------------------------------------------------------
int32_t oracle_csr_build(const int32_t* src, const int32_t* dst, const float* w, int64_t m,
                         int64_t num_nodes, uint32_t flags, int32_t offset_bits,
                         void* offsets_out, int32_t* nbrs_out, float* w_out,
                         int64_t* num_entries_out) {
  if (m < 0 || num_nodes < 0 || num_nodes > INT32_MAX) return ORACLE_EINVAL;
  if (offset_bits != 32 && offset_bits != 64) return ORACLE_EINVAL;
  if (m > 0 && (!src || !dst)) return ORACLE_EINVAL;
  if (!offsets_out || !num_entries_out) return ORACLE_EINVAL;
  if (w != nullptr && w_out == nullptr) return ORACLE_EINVAL;
  int64_t cap = (flags & ORACLE_SYMMETRIZE) ? 2 * m : m;
  if (offset_bits == 32 && cap > (int64_t)INT32_MAX) return ORACLE_EOVERFLOW;
  if (cap > 0 && !nbrs_out) return ORACLE_EINVAL;

  struct Entry { int32_t s, d; int64_t idx; };
  std::vector<Entry> e;
  e.reserve((size_t)cap);
  for (int64_t i = 0; i < m; ++i) {
    int32_t s = src[i], d = dst[i];
    if (s < 0 || d < 0 || s >= num_nodes || d >= num_nodes) continue;
    if ((flags & ORACLE_DROP_SELF_LOOPS) && s == d) continue;
    e.push_back(Entry{s, d, i});
    if (flags & ORACLE_SYMMETRIZE) e.push_back(Entry{d, s, i});
  }
  std::stable_sort(e.begin(), e.end(), [](const Entry& a, const Entry& b) {
    if (a.s != b.s) return a.s < b.s;
    if (a.d != b.d) return a.d < b.d;
    return a.idx < b.idx;
  });
  std::vector<int64_t> count((size_t)num_nodes + 1, 0);
  int64_t kept = 0;
  for (size_t i = 0; i < e.size(); ++i) {
    if ((flags & ORACLE_DEDUPE) && i > 0 && e[i].s == e[i - 1].s && e[i].d == e[i - 1].d)
      continue;
    nbrs_out[kept] = e[i].d;
    if (w != nullptr) w_out[kept] = w[e[i].idx];
    count[(size_t)e[i].s + 1] += 1;
    ++kept;
  }
  int64_t run = 0;
  for (int64_t v = 0; v <= num_nodes; ++v) {
    run += count[(size_t)v];
    if (offset_bits == 64) ((int64_t*)offsets_out)[v] = run;
    else ((int32_t*)offsets_out)[v] = (int32_t)run;
  }
  *num_entries_out = kept;
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Alias tables (Walker 1977; Vose 1991), one per segment.
// Segment s covers weights[seg_offsets[s] .. seg_offsets[s+1]).  With n entries
// and S = sum of the weights (added in index order, in fp64), entry i carries
// the scaled mass sc_i = w_i * n.  Entries with sc_i < S are "small", the rest
// "large"; both lists are first-in first-out and filled in index order.
// Repeatedly: take the oldest small a and the oldest large b; a keeps
// prob = sc_a / S of its own slot and the rest of the slot goes to b
// (alias[a] = b); b loses that much mass, sc_b = (sc_b + sc_a) - S, and is
// appended to the small or large list according to its new mass.
// Whatever remains in either list gets prob = 1 and aliases itself.
// alias[] holds positions inside the segment.
// ---------------------------------------------------------------------------
int32_t oracle_alias_build(const void* seg_offsets, int32_t offset_bits, int64_t num_segments,
                           const float* weights, float* prob_out, int32_t* alias_out) {
  if (offset_bits != 32 && offset_bits != 64) return ORACLE_EINVAL;
  if (num_segments < 0 || !seg_offsets) return ORACLE_EINVAL;
  std::vector<double> sc;
  std::deque<int64_t> small, large;
  for (int64_t s = 0; s < num_segments; ++s) {
    int64_t begin = offset_at(seg_offsets, offset_bits, s);
    int64_t end = offset_at(seg_offsets, offset_bits, s + 1);
    int64_t n = end - begin;
    if (n < 0) return ORACLE_EINVAL;
    if (n > (int64_t)INT32_MAX) return ORACLE_EOVERFLOW;
    if (n == 0) continue;
    const float* w = weights + begin;
    float* prob = prob_out + begin;
    int32_t* alias = alias_out + begin;
    double S = 0.0;
    for (int64_t i = 0; i < n; ++i) S += (double)w[i];
    sc.assign((size_t)n, 0.0);
    small.clear();
    large.clear();
    for (int64_t i = 0; i < n; ++i) {
      sc[(size_t)i] = (double)w[i] * (double)n;
      if (sc[(size_t)i] < S) small.push_back(i); else large.push_back(i);
    }
    while (!small.empty() && !large.empty()) {
      int64_t a = small.front(); small.pop_front();
      int64_t b = large.front(); large.pop_front();
      prob[a] = (float)(sc[(size_t)a] / S);
      alias[a] = (int32_t)b;
      sc[(size_t)b] = (sc[(size_t)b] + sc[(size_t)a]) - S;
      if (sc[(size_t)b] < S) small.push_back(b); else large.push_back(b);
    }
    for (int64_t i : small) { prob[i] = 1.0f; alias[i] = (int32_t)i; }
    for (int64_t i : large) { prob[i] = 1.0f; alias[i] = (int32_t)i; }
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// First-order walk (§2.2 DeepWalk: random walks from each node; §3.2: a walk
// contributes walk_len node ids to the batch, so walk_len counts nodes, the
// start included, and a walk makes walk_len - 1 transitions).
// Transition t of walk `id` uses the random block with counter
// (id low, id high, t, 0) under key `seed`.  Uniform: neighbour at
// slot(r64, deg).  Weighted: alias draw inside the row.  A node without
// out-edges ends the walk; the rest of the row is filled with -1.
// ---------------------------------------------------------------------------
int32_t oracle_random_walk(const oracle_csr* g, const oracle_alias* a, const int32_t* starts,
                           int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                           uint64_t seed, int32_t* walks_out) {
  if (!g || num_walks < 0 || walk_len < 1) return ORACLE_EINVAL;
  if (num_walks > 0 && (!starts || !walks_out)) return ORACLE_EINVAL;
  for (int64_t i = 0; i < num_walks; ++i) {
    int32_t* row = walks_out + i * (int64_t)walk_len;
    uint64_t id = walk_id_base + (uint64_t)i;
    int32_t v = starts[i];
    if (v < 0 || v >= g->num_nodes) v = -1;
    row[0] = v;
    for (int32_t t = 0; t + 1 < walk_len; ++t) {
      int32_t next = -1;
      if (v >= 0) {
        int64_t begin = offset_at(g->offsets, g->offset_bits, v);
        int64_t deg = offset_at(g->offsets, g->offset_bits, (int64_t)v + 1) - begin;
        if (deg > 0) {
          Block4 b = philox_keyed(seed, id, (uint32_t)t, 0u);
          next = g->nbrs[begin + draw_in_row(a, begin, deg, b)];
        }
      }
      row[t + 1] = next;
      v = next;
    }
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Second-order (node2vec) walk (§2.2: biased walk balancing breadth-first and
// depth-first exploration; Grover & Leskovec 2016 for the bias itself).
// The first transition has no previous node and is a first-order draw.
// Afterwards, with prev -> cur the last transition, a candidate x is drawn from
// the row of cur exactly as in the first-order walk and accepted with
// probability bias(x) / max_bias, where bias = 1/p if x == prev, 1 if prev has
// an edge to x, 1/q otherwise.  Attempt number `att` of transition t uses the
// block with counter (id low, id high, t, att); word 3 decides the acceptance:
// accept iff unit_float(word3) * max_bias < bias (one fp32 multiply, one
// compare).  Attempts are numbered 0..1023; the candidate of attempt 1023 is
// taken even if rejected, so the loop always ends.
// 1/p, 1/q and max_bias are computed once in fp32.
// ---------------------------------------------------------------------------
int32_t oracle_node2vec_walk(const oracle_csr* g, const oracle_alias* a, const int32_t* starts,
                             int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                             float p, float q, uint64_t seed, int32_t* walks_out) {
  if (!g || num_walks < 0 || walk_len < 1) return ORACLE_EINVAL;
  if (!(p > 0.0f) || !(q > 0.0f)) return ORACLE_EINVAL;
  if (num_walks > 0 && (!starts || !walks_out)) return ORACLE_EINVAL;
  const float inv_p = 1.0f / p;
  const float inv_q = 1.0f / q;
  const float max_bias = std::max(inv_p, std::max(1.0f, inv_q));
  for (int64_t i = 0; i < num_walks; ++i) {
    int32_t* row = walks_out + i * (int64_t)walk_len;
    uint64_t id = walk_id_base + (uint64_t)i;
    int32_t cur = starts[i];
    if (cur < 0 || cur >= g->num_nodes) cur = -1;
    int32_t prev = -1;
    row[0] = cur;
    for (int32_t t = 0; t + 1 < walk_len; ++t) {
      int32_t next = -1;
      if (cur >= 0) {
        int64_t begin = offset_at(g->offsets, g->offset_bits, cur);
        int64_t deg = offset_at(g->offsets, g->offset_bits, (int64_t)cur + 1) - begin;
        if (deg > 0) {
          for (uint32_t att = 0; att < 1024u; ++att) {
            Block4 b = philox_keyed(seed, id, (uint32_t)t, att);
            int32_t x = g->nbrs[begin + draw_in_row(a, begin, deg, b)];
            next = x;
            if (t == 0) break;  // no previous node yet
            float bias;
            if (x == prev) bias = inv_p;
            else if (row_contains(g, prev, x)) bias = 1.0f;
            else bias = inv_q;
            float scaled = unit_float(b.x[3]) * max_bias;
            if (scaled < bias) break;
          }
        }
      }
      row[t + 1] = next;
      prev = cur;
      cur = next;
    }
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Skip-gram pairs (§2.2: the skip-gram model applied to the walks; the window
// is the paper's "window-size").  For each walk in order, each position a of
// its valid prefix in order, each offset b = -W..W (b != 0) in ascending order
// with 0 <= a+b < len: emit (walk[a], walk[a+b]).  Fixed full window; nothing
// is subsampled or skipped, revisits of the centre included.
// ---------------------------------------------------------------------------
int32_t oracle_make_pairs(const int32_t* walks, int64_t num_walks, int32_t walk_len,
                          int32_t window, int32_t* centers_out, int32_t* contexts_out,
                          int64_t* num_pairs_out) {
  if (num_walks < 0 || walk_len < 1 || window < 1 || !num_pairs_out) return ORACLE_EINVAL;
  if (num_walks > 0 && !walks) return ORACLE_EINVAL;
  int64_t np = 0;
  for (int64_t i = 0; i < num_walks; ++i) {
    const int32_t* row = walks + i * (int64_t)walk_len;
    int32_t len = 0;
    while (len < walk_len && row[len] >= 0) ++len;
    for (int32_t pos = 0; pos < len; ++pos) {
      for (int32_t b = -window; b <= window; ++b) {
        if (b == 0) continue;
        int32_t other = pos + b;
        if (other < 0 || other >= len) continue;
        centers_out[np] = row[pos];
        contexts_out[np] = row[other];
        ++np;
      }
    }
  }
  *num_pairs_out = np;
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Negative samples (§2.2 "skip-gram and negative sampling"; §3.2 "negatively
// sampled nodes").  negs[i][k] is an alias draw from the single noise table of
// num_nodes entries, using the block with counter
// (pair index low, pair index high, k, 0x80000000).  Draws are independent:
// a negative equal to the centre or the context is kept.
// ---------------------------------------------------------------------------
int32_t oracle_sample_negatives(const oracle_alias* noise, int64_t num_nodes, int64_t num_pairs,
                                uint64_t pair_index_base, int32_t k, uint64_t seed,
                                int32_t* negs_out) {
  if (num_nodes < 1 || num_nodes > INT32_MAX || num_pairs < 0 || k < 0) return ORACLE_EINVAL;
  if (num_pairs > 0 && k > 0 && !negs_out) return ORACLE_EINVAL;
  for (int64_t i = 0; i < num_pairs; ++i) {
    uint64_t idx = pair_index_base + (uint64_t)i;
    for (int32_t j = 0; j < k; ++j) {
      Block4 b = philox_keyed(seed, idx, (uint32_t)j, 0x80000000u);
      negs_out[i * (int64_t)k + j] = (int32_t)draw_in_row(noise, 0, num_nodes, b);
    }
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// Edge sampling for LINE (§3.2: a LINE batch is B source nodes, one positive
// and num_neg negative nodes each; §4 trains LINE next to DeepWalk).  Sample i
// draws one CSR entry e with probability proportional to its weight (through an
// alias table over all entries, treated as one segment) or uniformly when no
// table is given, and returns (row that holds e, nbrs[e]).  In a symmetrised
// graph every undirected edge is present in both directions, so either endpoint
// can be the source.  Counter (sample index low, high, 0, 0x40000000).
// Rows without entries are never a source: the source of entry e is the one
// row r with offsets[r] <= e < offsets[r+1].
// ---------------------------------------------------------------------------
int32_t oracle_sample_edges(const oracle_csr* g, const oracle_alias* edge_alias, int64_t num_samples,
                            uint64_t sample_index_base, uint64_t seed, int32_t* centers_out,
                            int32_t* contexts_out) {
  if (!g || g->num_nodes < 1 || g->num_entries < 1 || num_samples < 0) return ORACLE_EINVAL;
  if (num_samples > 0 && (!centers_out || !contexts_out)) return ORACLE_EINVAL;
  std::vector<int32_t> source((size_t)g->num_entries);   // the row that holds each entry
  for (int64_t r = 0; r < g->num_nodes; ++r)
    for (int64_t e = offset_at(g->offsets, g->offset_bits, r);
         e < offset_at(g->offsets, g->offset_bits, r + 1); ++e)
      source[(size_t)e] = (int32_t)r;
  for (int64_t i = 0; i < num_samples; ++i) {
    Block4 b = philox_keyed(seed, sample_index_base + (uint64_t)i, 0u, 0x40000000u);
    const int64_t e = draw_in_row(edge_alias, 0, g->num_entries, b);
    centers_out[i] = source[(size_t)e];
    contexts_out[i] = g->nbrs[e];
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// One SGNS iteration (§3.2: loss on the batch's rows, gradient only for those
// rows, rows written back, barrier).  For pair i with u = W_in[c_i],
// v_0 = W_out[o_i], v_k = W_out[neg_{i,k}] (k = 1..K), x_j = <u, v_j>:
//   loss_i = softplus(-x_0) + sum_k softplus(x_k)
//   g_0 = sigmoid(x_0) - 1,  g_k = sigmoid(x_k)
//   dW_in[c_i]  += sum_j g_j v_j,   dW_out[row_j] += g_j u
// Every u and v is the value from before the call.  Afterwards each touched
// element becomes round(old - lr * d); loss_sum = sum_i loss_i.  Sums over
// pairs, not means.  All arithmetic in fp64, one rounding per written element.
// bf16 tables: elements are widened exactly on read and rounded to nearest
// even (through fp32) on write.
// ---------------------------------------------------------------------------
int32_t oracle_sgns_step(void* w_in, void* w_out, int64_t num_nodes, int32_t dim, int32_t dtype,
                         const int32_t* centers, const int32_t* contexts, const int32_t* negs,
                         int64_t num_pairs, int32_t k, float lr, double* loss_sum_out) {
  if (!w_in || !w_out || num_nodes < 1 || dim < 1 || num_pairs < 0 || k < 0) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  if (num_pairs > 0 && (!centers || !contexts || (k > 0 && !negs))) return ORACLE_EINVAL;
  if (!loss_sum_out) return ORACLE_EINVAL;
  RowSums d_in, d_out;
  int32_t rc = sgns_gradients(w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs, num_pairs,
                              k, d_in, d_out, loss_sum_out);
  if (rc != ORACLE_OK) return rc;
  const double step = (double)lr;
  for (auto& kv : d_in)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(w_in, dtype, dim, kv.first, e,
                 read_elem(w_in, dtype, dim, kv.first, e) - step * kv.second[(size_t)e]);
  for (auto& kv : d_out)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(w_out, dtype, dim, kv.first, e,
                 read_elem(w_out, dtype, dim, kv.first, e) - step * kv.second[(size_t)e]);
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// The same iteration with the optimizer the paper runs (§3.2, model update for
// SGD with momentum as three storage operations), for both tables:
//   mult      momentum <- mu * momentum                 (every row)
//   put       momentum[r] <- momentum[r] + gradient[r]  (rows of the batch)
//   mult_add  model <- model - lr * momentum            (every row)
// The gradient is that of the batch's summed SGNS loss at the pre-iteration
// model.  Each operation reads stored values and rounds once on writing.
// ---------------------------------------------------------------------------
int32_t oracle_sgns_momentum_step(void* w_in, void* w_out, void* m_in, void* m_out,
                                  int64_t num_nodes, int32_t dim, int32_t dtype,
                                  const int32_t* centers, const int32_t* contexts,
                                  const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                  float mu, double* loss_sum_out) {
  if (!w_in || !w_out || !m_in || !m_out || num_nodes < 1 || dim < 1 || num_pairs < 0 || k < 0)
    return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  if (num_pairs > 0 && (!centers || !contexts || (k > 0 && !negs))) return ORACLE_EINVAL;
  if (!loss_sum_out) return ORACLE_EINVAL;
  RowSums d_in, d_out;
  int32_t rc = sgns_gradients(w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs, num_pairs,
                              k, d_in, d_out, loss_sum_out);
  if (rc != ORACLE_OK) return rc;
  void* model[2] = {w_in, w_out};
  void* moment[2] = {m_in, m_out};
  RowSums* grad[2] = {&d_in, &d_out};
  for (int tb = 0; tb < 2; ++tb) {
    for (int64_t r = 0; r < num_nodes; ++r)
      for (int32_t e = 0; e < dim; ++e)
        write_elem(moment[tb], dtype, dim, r, e, (double)mu * read_elem(moment[tb], dtype, dim, r, e));
    for (auto& kv : *grad[tb])
      for (int32_t e = 0; e < dim; ++e)
        write_elem(moment[tb], dtype, dim, kv.first, e,
                   read_elem(moment[tb], dtype, dim, kv.first, e) + kv.second[(size_t)e]);
    for (int64_t r = 0; r < num_nodes; ++r)
      for (int32_t e = 0; e < dim; ++e)
        write_elem(model[tb], dtype, dim, r, e,
                   read_elem(model[tb], dtype, dim, r, e) -
                       (double)lr * read_elem(moment[tb], dtype, dim, r, e));
  }
  return ORACLE_OK;
}


// ---------------------------------------------------------------------------
// LINE with first-order proximity (the LINE paper the text cites in §2.2 / §4):
// one table w on both sides.  For sampled edge (s, t) and negatives n_k:
//   x_0 = <w[s], w[t]>, x_k = <w[s], w[n_k]>, loss and g as in the SGNS step;
//   gradient of w[s] += sum_j g_j w[row_j], gradient of w[row_j] += g_j w[s]
// (a row gets both kinds of contribution when it appears on both sides), all
// from the values before the call.  The rows are then written in two rounds,
// each rounding once: first the contributions a row receives as target or
// negative, then those it receives as source.
// ---------------------------------------------------------------------------
int32_t oracle_line1_step(void* w, int64_t num_nodes, int32_t dim, int32_t dtype,
                          const int32_t* sources, const int32_t* targets, const int32_t* negs,
                          int64_t num_pairs, int32_t k, float lr, double* loss_sum_out) {
  if (!w || num_nodes < 1 || dim < 1 || num_pairs < 0 || k < 0 || !loss_sum_out) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  if (num_pairs > 0 && (!sources || !targets || (k > 0 && !negs))) return ORACLE_EINVAL;
  RowSums as_source, as_other;
  int32_t rc = sgns_gradients(w, w, num_nodes, dim, dtype, sources, targets, negs, num_pairs, k,
                              as_source, as_other, loss_sum_out);
  if (rc != ORACLE_OK) return rc;
  const double step = (double)lr;
  for (auto& kv : as_other)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(w, dtype, dim, kv.first, e,
                 read_elem(w, dtype, dim, kv.first, e) - step * kv.second[(size_t)e]);
  for (auto& kv : as_source)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(w, dtype, dim, kv.first, e,
                 read_elem(w, dtype, dim, kv.first, e) - step * kv.second[(size_t)e]);
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// The same iteration with Adam (§3.2 names Adam next to SGD with momentum as an
// optimizer kept inside the storage; the update rule is Kingma & Ba's), run the
// same way as the momentum step: dense operations over every row around a sparse
// put of the batch's gradient rows g (zero for rows outside the batch):
//   mult   m <- beta1 * m,  v <- beta2 * v                               (every row)
//   put    m[r] <- m[r] + (1 - beta1) * g[r],  v[r] <- v[r] + (1 - beta2) * g[r]^2
//   apply  w <- w - (lr / (1 - beta1^t)) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps)
// t >= 1 is the number of this iteration.  Each operation reads stored values
// and rounds once on writing.  fp32 tables only.
// ---------------------------------------------------------------------------
int32_t oracle_sgns_adam_step(float* w_in, float* w_out, float* m_in, float* m_out, float* v_in,
                              float* v_out, int64_t num_nodes, int32_t dim, const int32_t* centers,
                              const int32_t* contexts, const int32_t* negs, int64_t num_pairs,
                              int32_t k, float lr, float beta1, float beta2, float eps, int64_t t,
                              double* loss_sum_out) {
  if (!w_in || !w_out || !m_in || !m_out || !v_in || !v_out || t < 1) return ORACLE_EINVAL;
  if (num_nodes < 1 || dim < 1 || num_pairs < 0 || k < 0 || !loss_sum_out) return ORACLE_EINVAL;
  if (num_pairs > 0 && (!centers || !contexts || (k > 0 && !negs))) return ORACLE_EINVAL;
  RowSums d_in, d_out;
  int32_t rc = sgns_gradients(w_in, w_out, num_nodes, dim, ORACLE_F32, centers, contexts, negs,
                              num_pairs, k, d_in, d_out, loss_sum_out);
  if (rc != ORACLE_OK) return rc;
  const double b1 = (double)beta1, b2 = (double)beta2;
  const double step = (double)lr / (1.0 - std::pow(b1, (double)t));
  const double root_c2 = std::sqrt(1.0 - std::pow(b2, (double)t));
  float* model[2] = {w_in, w_out};
  float* first[2] = {m_in, m_out};
  float* second[2] = {v_in, v_out};
  RowSums* grad[2] = {&d_in, &d_out};
  for (int tb = 0; tb < 2; ++tb) {
    const int64_t total = num_nodes * (int64_t)dim;
    for (int64_t i = 0; i < total; ++i) {
      first[tb][i] = (float)(b1 * (double)first[tb][i]);
      second[tb][i] = (float)(b2 * (double)second[tb][i]);
    }
    for (auto& kv : *grad[tb])
      for (int32_t e = 0; e < dim; ++e) {
        const int64_t i = kv.first * (int64_t)dim + e;
        const double g = kv.second[(size_t)e];
        first[tb][i] = (float)((double)first[tb][i] + (1.0 - b1) * g);
        second[tb][i] = (float)((double)second[tb][i] + (1.0 - b2) * g * g);
      }
    for (int64_t i = 0; i < total; ++i) {
      const double m = (double)first[tb][i], v = (double)second[tb][i];
      model[tb][i] = (float)((double)model[tb][i] - step * m / (std::sqrt(v) / root_c2 + (double)eps));
    }
  }
  return ORACLE_OK;
}

// ---------------------------------------------------------------------------
// The storage operations of §3.1 / §3.2 on a batch of vertex ids: a trainer
// merges equal ids of its batch into one request, fetches one n x d block of
// rows (get), and sends back one block of gradient rows that the storage adds
// to its rows (put).
//
// unique: the distinct ids of the batch in ascending order, and for every
// batch entry the position of its id in that list.  Ids outside [0, num_nodes)
// belong to no row: they are left out and their position is -1.
// ---------------------------------------------------------------------------
int32_t oracle_unique_ids(const int32_t* ids, int64_t n, int64_t num_nodes, int32_t* unique_out,
                          int64_t* num_unique_out, int32_t* inverse_out) {
  if (n < 0 || num_nodes < 1 || !num_unique_out || (n > 0 && (!ids || !unique_out)))
    return ORACLE_EINVAL;
  std::vector<int32_t> sorted;
  for (int64_t i = 0; i < n; ++i)
    if (ids[i] >= 0 && (int64_t)ids[i] < num_nodes) sorted.push_back(ids[i]);
  std::sort(sorted.begin(), sorted.end());
  sorted.erase(std::unique(sorted.begin(), sorted.end()), sorted.end());
  for (size_t j = 0; j < sorted.size(); ++j) unique_out[j] = sorted[j];
  *num_unique_out = (int64_t)sorted.size();
  if (inverse_out)
    for (int64_t i = 0; i < n; ++i) {
      auto it = std::lower_bound(sorted.begin(), sorted.end(), ids[i]);
      inverse_out[i] = (it != sorted.end() && *it == ids[i]) ? (int32_t)(it - sorted.begin()) : -1;
    }
  return ORACLE_OK;
}

// get: out[i] = table[ids[i]] as fp32 (bf16 widened exactly); a zero row for an
// id outside [0, num_nodes).
int32_t oracle_get_rows(const void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                        const int32_t* ids, int64_t n, float* out) {
  if (!table || num_nodes < 1 || dim < 1 || n < 0 || (n > 0 && (!ids || !out))) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  for (int64_t i = 0; i < n; ++i)
    for (int32_t e = 0; e < dim; ++e) {
      const bool ok = ids[i] >= 0 && (int64_t)ids[i] < num_nodes;
      out[i * (int64_t)dim + e] = ok ? (float)read_elem(table, dtype, dim, ids[i], e) : 0.0f;
    }
  return ORACLE_OK;
}

// put: table[ids[i]] <- round(table[ids[i]] + scale * rows[i]), ids distinct
// (an id outside [0, num_nodes) is skipped).  One rounding per element.
int32_t oracle_put_rows(void* table, int64_t num_nodes, int32_t dim, int32_t dtype, const int32_t* ids,
                        int64_t n, const float* rows, float scale) {
  if (!table || num_nodes < 1 || dim < 1 || n < 0 || (n > 0 && (!ids || !rows))) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  std::vector<int32_t> seen(ids, ids + n);
  std::sort(seen.begin(), seen.end());
  for (size_t j = 1; j < seen.size(); ++j)
    if (seen[j] == seen[j - 1] && seen[j] >= 0 && (int64_t)seen[j] < num_nodes) return ORACLE_EINVAL;
  for (int64_t i = 0; i < n; ++i) {
    if (ids[i] < 0 || (int64_t)ids[i] >= num_nodes) continue;
    for (int32_t e = 0; e < dim; ++e)
      write_elem(table, dtype, dim, ids[i], e,
                 read_elem(table, dtype, dim, ids[i], e) + (double)scale * (double)rows[i * (int64_t)dim + e]);
  }
  return ORACLE_OK;
}


// The two dense storage operations of §3.2 (model update for SGD with momentum):
// mult: every element of a table times a factor; mult_add: dst <- dst + factor * src
// for two tables of the same shape.  One rounding per element.
int32_t oracle_table_mult(void* table, int64_t num_nodes, int32_t dim, int32_t dtype, float factor) {
  if (!table || num_nodes < 1 || dim < 1) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  for (int64_t r = 0; r < num_nodes; ++r)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(table, dtype, dim, r, e, (double)factor * read_elem(table, dtype, dim, r, e));
  return ORACLE_OK;
}

int32_t oracle_table_mult_add(void* dst, const void* src, int64_t num_nodes, int32_t dim,
                              int32_t dtype, float factor) {
  if (!dst || !src || num_nodes < 1 || dim < 1) return ORACLE_EINVAL;
  if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F16) return ORACLE_EINVAL;
  for (int64_t r = 0; r < num_nodes; ++r)
    for (int32_t e = 0; e < dim; ++e)
      write_elem(dst, dtype, dim, r, e,
                 read_elem(dst, dtype, dim, r, e) + (double)factor * read_elem(src, dtype, dim, r, e));
  return ORACLE_OK;
}


// Reorders a batch of (centre, context) pairs by centre id, keeping the input
// order among pairs of equal centre (a stable sort).  The order of the pairs
// inside a batch does not change an iteration's result (sums over the batch);
// equal centres next to each other let the step load and write a centre row
// once per run.  Ids outside [0, num_nodes) go last, in input order.
int32_t oracle_sort_pairs(const int32_t* centers, const int32_t* contexts, int64_t n,
                          int64_t num_nodes, int32_t* centers_out, int32_t* contexts_out) {
  if (n < 0 || num_nodes < 1 || (n > 0 && (!centers || !contexts || !centers_out || !contexts_out)))
    return ORACLE_EINVAL;
  std::vector<int64_t> order((size_t)n);
  for (int64_t i = 0; i < n; ++i) order[(size_t)i] = i;
  auto key = [&](int64_t i) -> int64_t {
    return (centers[i] >= 0 && (int64_t)centers[i] < num_nodes) ? (int64_t)centers[i] : num_nodes;
  };
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return key(a) < key(b); });
  for (int64_t j = 0; j < n; ++j) {
    centers_out[j] = centers[order[(size_t)j]];
    contexts_out[j] = contexts[order[(size_t)j]];
  }
  return ORACLE_OK;
}


// binary16 conversions, exported for their pins
void oracle_f16_to_float(const uint16_t* in, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = f16_to_float(in[i]);
}
void oracle_float_to_f16(const float* in, int64_t n, uint16_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = float_to_f16(in[i]);
}

}  // extern "C"
