// gs_random_walk / gs_node2vec_walk (GraphScale Sec. 2.2: DeepWalk-style walks
// from every node and node2vec's biased second-order walk).
//
// One lane per walk.  Every transition is a chain of dependent random reads
// (row bounds -> neighbour -> for node2vec, the previous node's row), each of
// which costs a whole cache line from HBM, so throughput comes from many walks
// in flight and from touching few lines per step.  Output rows are staged in LDS
// in windows of kWin positions and written out as 64-byte row segments instead
// of one scattered 4-byte store per position.
#include "common.h"

namespace gs {

constexpr int kWalkThreads = 256;
constexpr int kWin = 16;          // positions staged per flush
constexpr int kWinPad = kWin + 1; // odd stride: conflict-free column writes
constexpr uint32_t kMaxAttempts = 1024;

struct WalkArgs {
  const void* offsets;
  const int32_t* nbrs;
  const float* prob;
  const int32_t* alias;
  const uint2* packed;      // optional interleaved (prob bits, alias)
  const int32_t* starts;
  int32_t* walks;
  int64_t num_nodes;
  int64_t num_entries;
  int64_t num_walks;
  uint64_t id_base;
  uint64_t seed;
  int32_t walk_len;
  float inv_p, inv_q, max_bias;
};

// Alias step of a weighted draw: keep slot j, or move to the slot's alias.
__device__ __forceinline__ int64_t alias_pick(const WalkArgs& a, int64_t at, int64_t j, uint32_t word) {
  if (a.packed != nullptr) {
    const uint2 e = a.packed[at];
    return (unit_float(word) < __uint_as_float(e.x)) ? j : (int64_t)(int32_t)e.y;
  }
  return (unit_float(word) < a.prob[at]) ? j : (int64_t)a.alias[at];
}

// First-order walks: one lane per walk, one dependent pair of random reads per
// step (row bounds, then the neighbour).  The 64 walks of a wave advance in
// lock step, so their positions are staged in LDS in windows of kWin and the
// wave writes them out together, 64 bytes per row segment.
template <typename OffT, bool kWeighted>
__global__ __launch_bounds__(kWalkThreads) void walk_kernel(WalkArgs a) {
  __shared__ int32_t tile[kWalkThreads / 64][64][kWinPad];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t wave_first = ((int64_t)blockIdx.x * (kWalkThreads / 64) + wave) * 64;
  const int64_t i = wave_first + lane;
  const bool live = i < a.num_walks;
  const uint64_t id = a.id_base + (uint64_t)i;
  const int32_t* __restrict__ nbrs = a.nbrs;
  const OffT* __restrict__ offsets = static_cast<const OffT*>(a.offsets);

  int32_t cur = -1;
  if (live) {
    cur = a.starts[i];
    if (cur < 0 || (int64_t)cur >= a.num_nodes) cur = -1;
  }

  for (int32_t t0 = 0; t0 < a.walk_len; t0 += kWin) {
    const int cols = min(kWin, a.walk_len - t0);
    for (int tt = 0; tt < cols; ++tt) {
      const int32_t t = t0 + tt;
      tile[wave][lane][tt] = cur;
      if (t + 1 >= a.walk_len) break;
      int32_t next = -1;
      if (cur >= 0) {
        const int64_t lo = (int64_t)offsets[cur];
        const int64_t hi = (int64_t)offsets[(int64_t)cur + 1];
        if (hi > lo) {
          const Block4 b = philox_at(a.seed, id, (uint32_t)t, 0u);
          int64_t j = (int64_t)slot_of(b, (uint64_t)(hi - lo));
          if (kWeighted) {
            j = alias_pick(a, lo + j, j, b.x2);
          }
          next = nbrs[lo + j];
          // a neighbour id that is not a node (a CSR not built by gs_csr_build) ends the walk
          if ((uint32_t)next >= (uint32_t)a.num_nodes) next = -1;
        }
      }
      cur = next;
    }
    __syncthreads();
    // flush: 4 rows per pass, 16 lanes (64 bytes) per row
    const int c = lane & 15;
#pragma unroll 4
    for (int pass = 0; pass < 16; ++pass) {
      const int r = pass * 4 + (lane >> 4);
      const int64_t w = wave_first + r;
      if (w < a.num_walks && c < cols)
        a.walks[w * (int64_t)a.walk_len + t0 + c] = tile[wave][r][c];
    }
    __syncthreads();
  }
}

// Second-order walks as a per-lane state machine with ONE memory access per
// loop iteration.  A step of a walk is a chain of dependent random reads of
// very different length (row bounds; one candidate per attempt, 3.5 attempts on
// average at p=0.5, q=2; for a quarter of the attempts a search in the previous
// node's row).  Written as nested loops, a wave waits in every inner loop for
// its slowest lane and keeps about a third of its lanes busy.  Here every lane
// carries its own state (which read it needs next), each iteration issues that
// one read for all 64 lanes together, and the lane then moves to its next state;
// lanes never wait for each other except at the one load per iteration.
// The membership search in the previous node's row is an interpolation search (the ids of
// a row are spread evenly over [0, num_nodes), so x is expected where a straight line
// between the entries that bound the remaining range puts it; every third probe bisects
// instead, which bounds the search on rows that are not spread evenly).  A probe reads four
// neighbouring entries (one 16-byte access, the same cache line as a 4-byte one), and a
// probe whose entries lie on both sides of x ends the search at once.
// Each lane stages its own last kWin positions in LDS and writes them out as one
// 64-byte row segment when the window is full (or the walk is over).
struct __attribute__((packed, aligned(4))) Quad { int32_t v[4]; };   // four entries, 4-byte aligned
template <typename OffT, bool kWeighted>
__global__ __launch_bounds__(kWalkThreads) void node2vec_kernel(WalkArgs a) {
  __shared__ int32_t tile[kWalkThreads / 64][64][kWinPad];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t i = ((int64_t)blockIdx.x * (kWalkThreads / 64) + wave) * 64 + lane;
  if (i >= a.num_walks) return;
  const uint64_t id = a.id_base + (uint64_t)i;
  const int32_t* __restrict__ nbrs = a.nbrs;
  const OffT* __restrict__ offsets = static_cast<const OffT*>(a.offsets);
  int32_t* __restrict__ out = a.walks + i * (int64_t)a.walk_len;
  int32_t* mine = tile[wave][lane];
  const int32_t last = a.walk_len - 1;      // index of the last position
  const float bias_lo = fminf(1.0f, a.inv_q), bias_hi = fmaxf(1.0f, a.inv_q);

  enum : int { kRow, kNewDraw, kAlias, kDraw, kSearch, kDone };
  enum : int { kNone, kCommit, kReject };
  const bool wide = a.num_entries >= 4;     // (a probe never reads past the array)
  int32_t cur = a.starts[i];
  if (cur < 0 || (int64_t)cur >= a.num_nodes) cur = -1;
  int32_t prev = -1;
  int64_t prev_lo = 0, prev_hi = 0, lo = 0, hi = 0;
  int32_t t = 0;                            // position of cur
  uint32_t att = 0;
  int state = kRow;
  int decision = kNone;                     // what the last read decided: taken at the top of the loop
  int32_t next = -1;                        // the node a commit moves to
  mine[0] = cur;
  if (last == 0) { out[0] = cur; return; }

  // the attempt in flight
  int64_t j = 0;                            // slot in the row of cur
  uint32_t word2 = 0;                       // alias uniform (weighted)
  float s = 0.f;                            // acceptance uniform * max_bias
  int32_t x = 0;                            // candidate
  // the membership search in flight: entries before L are < x, entries from H on are > x;
  // v_lo < x is the entry before L (or -1), v_hi > x the entry at H (or num_nodes)
  int64_t L = 0, H = 0;
  int32_t v_lo = 0, v_hi = 0;
  int probes = 0;                           // probes made in this search
  int64_t pos = 0;                          // what this iteration reads: nbrs[pos] (or the alias entry at pos)

  // position t + 1 of the walk is `node`: into the lane's window, and out when it is full
  auto put = [&](int32_t node) {
    ++t;
    const int col = t & (kWin - 1);
    mine[col] = node;
    if (col == kWin - 1 || t == last) {
      const int32_t first = t - col;
      for (int c = 0; c <= col; ++c) out[first + c] = mine[c];
    }
  };

  // Every stage below appears once, so a wave whose lanes are in different states runs each
  // of them once per trip: the decision of the last read (a step taken, or an attempt
  // rejected), the random numbers of a new attempt, the address of the next read, the read,
  // and what the value read means for the lane's state.
  while (true) {
    // ---- the decision of the last read ----------------------------------------------------
    if (decision == kCommit) {
      prev = cur; prev_lo = lo; prev_hi = hi;
      cur = next;
      att = 0;
      put(cur);
      state = (t == last) ? kDone : kRow;
    } else if (decision == kReject) {
      ++att;
      state = kNewDraw;
    }
    decision = kNone;
    if (state == kRow && cur < 0) {          // dead walk: -1 to the end
      while (t < last) put(-1);
      state = kDone;
    }
    if (state == kDone) break;

    // ---- arithmetic ahead of the read -----------------------------------------------------
    if (state == kNewDraw) {
      const Block4 b = philox_at(a.seed, id, (uint32_t)t, att);
      j = (int64_t)slot_of(b, (uint64_t)(hi - lo));
      word2 = b.x2;
      s = unit_float(b.x3) * a.max_bias;
      pos = lo + j;
      state = (kWeighted ? kAlias : kDraw);
    } else if (state == kSearch) {           // (the range [L, H) is never empty here)
      int64_t p;
      if (probes % 3 == 2) {
        p = L + ((H - L) >> 1);
      } else {
        const float part = (float)((int64_t)x - v_lo) / (float)((int64_t)v_hi - v_lo);
        p = L + (int64_t)(part * (float)(H - L));
      }
      p = min(max(p, L), H - 1);
      // the four entries around p: an aligned group, or the array's last four
      pos = wide ? min(p & ~(int64_t)3, a.num_entries - 4) : p;
    }

    // ---- the one read of this iteration ---------------------------------------------------
    int64_t r0 = 0, r1 = 0;
    int32_t v = 0;
    Quad quad = {{0, 0, 0, 0}};
    uint32_t e_prob = 0, e_alias = 0;
    if (state == kSearch) {
      if (wide) quad = *reinterpret_cast<const Quad*>(nbrs + pos);
      else quad.v[0] = nbrs[pos];
    } else if (state == kRow) {
      r0 = (int64_t)offsets[cur];
      r1 = (int64_t)offsets[(int64_t)cur + 1];
    } else if (kWeighted && state == kAlias) {
      if (a.packed != nullptr) { const uint2 e = a.packed[pos]; e_prob = e.x; e_alias = e.y; }
      else { e_prob = __float_as_uint(a.prob[pos]); e_alias = (uint32_t)a.alias[pos]; }
    } else {
      v = nbrs[pos];
    }

    // ---- consume it: new state, or a decision ----------------------------------------------
    bool known = false, member = false;      // membership of x in the row of prev has been settled
    switch (state) {
      case kRow:
        lo = r0; hi = r1;
        if (hi > lo) state = kNewDraw;
        else { decision = kCommit; next = -1; }                    // dead end
        break;
      case kAlias:
        if (!(unit_float(word2) < __uint_as_float(e_prob))) j = (int64_t)(int32_t)e_alias;
        pos = lo + j;
        state = kDraw;
        break;
      case kDraw:
        x = v;
        next = x;
        // a neighbour id that is not a node (a CSR not built by gs_csr_build) ends the walk
        if ((uint32_t)x >= (uint32_t)a.num_nodes) { decision = kCommit; next = -1; break; }
        if (t == 0 || att == kMaxAttempts - 1) { decision = kCommit; break; }   // unbiased first step; last attempt is taken
        // accept iff s < bias(x).  For x != prev the bias is 1 or 1/q, so the
        // membership search is only needed when s falls between the two.
        if (x == prev) { decision = (s < a.inv_p) ? kCommit : kReject; break; }
        if (s < bias_lo) { decision = kCommit; break; }
        if (!(s < bias_hi)) { decision = kReject; break; }
        L = prev_lo; H = prev_hi;
        if (L >= H) { known = true; break; }                       // (prev has no row: cannot happen after a step)
        v_lo = -1;
        v_hi = (int32_t)a.num_nodes;
        probes = 0;
        state = kSearch;
        break;
      case kSearch: {
        // entries pos + i0 .. pos + i1 of the probe lie in the remaining range [L, H)
        const int width = wide ? 4 : 1;
        const int i0 = (int)(max(pos, L) - pos), i1 = (int)(min(pos + width, H) - 1 - pos);
        bool found = false;
        int32_t first_v = 0, last_v = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          found = found || (q >= i0 && q <= i1 && quad.v[q] == x);
          if (q == i0) first_v = quad.v[q];
          if (q == i1) last_v = quad.v[q];
        }
        ++probes;
        if (found) { known = true; member = true; break; }
        if (x < first_v) { H = pos + i0; v_hi = first_v; }
        else if (x > last_v) { L = pos + i1 + 1; v_lo = last_v; }
        else known = true;                  // x lies between two neighbouring entries
        if (L >= H) known = true;
        break;
      }
      default:
        break;
    }
    if (known) decision = (s < (member ? 1.0f : a.inv_q)) ? kCommit : kReject;
  }
}

template <typename OffT>
static void launch_walk(bool weighted, bool second, const WalkArgs& a, hipStream_t stream) {
  const unsigned blocks = (unsigned)ceil_div(a.num_walks, kWalkThreads);
  if (second) {
    if (weighted) node2vec_kernel<OffT, true><<<blocks, kWalkThreads, 0, stream>>>(a);
    else node2vec_kernel<OffT, false><<<blocks, kWalkThreads, 0, stream>>>(a);
  } else {
    if (weighted) walk_kernel<OffT, true><<<blocks, kWalkThreads, 0, stream>>>(a);
    else walk_kernel<OffT, false><<<blocks, kWalkThreads, 0, stream>>>(a);
  }
}

static int32_t walk_common(const gs_csr* g, const gs_alias* al, const int32_t* starts,
                           int64_t num_walks, uint64_t id_base, int32_t walk_len, bool second,
                           float p, float q, uint64_t seed, int32_t* walks_out, hipStream_t stream) {
  if (!g || num_walks < 0 || walk_len < 1) return GS_EINVAL;
  if (g->num_nodes < 0 || g->num_nodes > (int64_t)INT32_MAX || g->num_entries < 0) return GS_EINVAL;
  if (g->offset_bits != 32 && g->offset_bits != 64) return GS_EINVAL;
  if (!g->offsets || (g->num_entries > 0 && !g->nbrs)) return GS_EINVAL;
  if (second && (!(p > 0.0f) || !(q > 0.0f))) return GS_EINVAL;
  if (num_walks > 0 && (!starts || !walks_out)) return GS_EINVAL;
  if (num_walks > ((int64_t)1 << 38)) return GS_EOVERFLOW;
  const bool weighted = al != nullptr && al->prob != nullptr;
  if (weighted && !al->alias) return GS_EINVAL;
  if (num_walks == 0) return GS_OK;
  WalkArgs a;
  a.offsets = g->offsets;
  a.nbrs = g->nbrs;
  a.prob = weighted ? al->prob : nullptr;
  a.alias = weighted ? al->alias : nullptr;
  a.packed = weighted ? reinterpret_cast<const uint2*>(al->packed) : nullptr;
  a.starts = starts;
  a.walks = walks_out;
  a.num_nodes = g->num_nodes;
  a.num_entries = g->num_entries;
  a.num_walks = num_walks;
  a.id_base = id_base;
  a.seed = seed;
  a.walk_len = walk_len;
  a.inv_p = 1.0f / p;
  a.inv_q = 1.0f / q;
  a.max_bias = fmaxf(a.inv_p, fmaxf(1.0f, a.inv_q));
  if (g->offset_bits == 64) launch_walk<int64_t>(weighted, second, a, stream);
  else launch_walk<int32_t>(weighted, second, a, stream);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

}  // namespace gs

extern "C" int32_t gs_random_walk(const gs_csr* g, const gs_alias* a, const int32_t* starts,
                                  int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                                  uint64_t seed, int32_t* walks_out, void* stream) {
  return gs::walk_common(g, a, starts, num_walks, walk_id_base, walk_len, false, 1.0f, 1.0f, seed,
                         walks_out, (hipStream_t)stream);
}

extern "C" int32_t gs_node2vec_walk(const gs_csr* g, const gs_alias* a, const int32_t* starts,
                                    int64_t num_walks, uint64_t walk_id_base, int32_t walk_len,
                                    float p, float q, uint64_t seed, int32_t* walks_out,
                                    void* stream) {
  return gs::walk_common(g, a, starts, num_walks, walk_id_base, walk_len, true, p, q, seed,
                         walks_out, (hipStream_t)stream);
}
