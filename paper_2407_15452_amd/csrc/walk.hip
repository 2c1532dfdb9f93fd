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
  int64_t num_walks;
  uint64_t id_base;
  uint64_t seed;
  int32_t walk_len;
  float inv_p, inv_q, max_bias;
  float inv_num_nodes;
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
// Each lane stages its own last kWin positions in LDS and writes them out as one
// 64-byte row segment when the window is full (or the walk is over).
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

  enum : int { kRow, kNewDraw, kAlias, kDraw, kProbe1, kProbe2, kGallop, kBinary, kDone };
  int32_t cur = a.starts[i];
  if (cur < 0 || (int64_t)cur >= a.num_nodes) cur = -1;
  int32_t prev = -1;
  int64_t prev_lo = 0, prev_hi = 0, lo = 0, hi = 0;
  int32_t t = 0;                            // position of cur
  uint32_t att = 0;
  int state = kRow;
  mine[0] = cur;
  if (last == 0) { out[0] = cur; return; }

  // the attempt in flight
  int64_t j = 0;                            // slot in the row of cur
  uint32_t word2 = 0;                       // alias uniform (weighted)
  float s = 0.f;                            // acceptance uniform * max_bias
  int32_t x = 0;                            // candidate
  // the membership search in flight: entries before L are < x, entries from H on are > x
  int64_t L = 0, H = 0, p = 0, step = 1;
  float slope = 0.f;
  bool right = false;
  int64_t pos = 0;                          // what this iteration reads: nbrs[pos] (or the alias entry at pos)

  auto commit = [&](int32_t next) {         // the step is decided: move to position t + 1
    prev = cur; prev_lo = lo; prev_hi = hi;
    cur = next;
    ++t;
    att = 0;
    const int col = t & (kWin - 1);
    mine[col] = cur;
    if (col == kWin - 1 || t == last) {
      const int32_t first = t - col;
      for (int c = 0; c <= col; ++c) out[first + c] = mine[c];
    }
    state = (t == last) ? kDone : kRow;
  };
  auto reject = [&]() { ++att; state = kNewDraw; };
  auto resolve = [&](bool member) {         // membership of x in the row of prev is known
    if (s < (member ? 1.0f : a.inv_q)) commit(x); else reject();
  };

  while (state != kDone) {
    // ---- bring the lane to a state that needs a read (arithmetic only) -------------------
    bool ready = false;
    while (!ready) {
      switch (state) {
        case kRow:
          if (cur < 0) { while (state != kDone) commit(-1); }   // dead walk: -1 to the end
          ready = true;
          break;
        case kNewDraw: {
          const Block4 b = philox_at(a.seed, id, (uint32_t)t, att);
          j = (int64_t)slot_of(b, (uint64_t)(hi - lo));
          word2 = b.x2;
          s = unit_float(b.x3) * a.max_bias;
          pos = lo + j;
          state = (kWeighted ? kAlias : kDraw);
          ready = true;
          break;
        }
        case kGallop:
          if (L >= H) { resolve(false); break; }
          pos = right ? min(L + step - 1, H - 1) : max(H - step, L);
          ready = true;
          break;
        case kBinary:
          if (L >= H) { resolve(false); break; }
          pos = L + ((H - L) >> 1);
          ready = true;
          break;
        default:                            // kAlias, kDraw, kProbe1, kProbe2, kDone: pos is set
          ready = true;
          break;
      }
    }
    if (state == kDone) break;

    // ---- the one read of this iteration ---------------------------------------------------
    int64_t r0 = 0, r1 = 0;
    int32_t v = 0;
    uint32_t e_prob = 0, e_alias = 0;
    if (state == kRow) {
      r0 = (int64_t)offsets[cur];
      r1 = (int64_t)offsets[(int64_t)cur + 1];
    } else if (kWeighted && state == kAlias) {
      if (a.packed != nullptr) { const uint2 e = a.packed[pos]; e_prob = e.x; e_alias = e.y; }
      else { e_prob = __float_as_uint(a.prob[pos]); e_alias = (uint32_t)a.alias[pos]; }
    } else {
      v = nbrs[pos];
    }

    // ---- consume it --------------------------------------------------------------------------
    switch (state) {
      case kRow:
        lo = r0; hi = r1;
        if (hi > lo) state = kNewDraw; else commit(-1);           // dead end
        break;
      case kAlias:
        if (!(unit_float(word2) < __uint_as_float(e_prob))) j = (int64_t)(int32_t)e_alias;
        pos = lo + j;
        state = kDraw;
        break;
      case kDraw:
        x = v;
        // a neighbour id that is not a node (a CSR not built by gs_csr_build) ends the walk
        if ((uint32_t)x >= (uint32_t)a.num_nodes) { commit(-1); break; }
        if (t == 0 || att == kMaxAttempts - 1) { commit(x); break; }   // unbiased first step; last attempt is taken
        // accept iff s < bias(x).  For x != prev the bias is 1 or 1/q, so the
        // membership search is only needed when s falls between the two.
        if (x == prev) { if (s < a.inv_p) commit(x); else reject(); break; }
        if (s < bias_lo) { commit(x); break; }
        if (!(s < bias_hi)) { reject(); break; }
        L = prev_lo; H = prev_hi;
        if (H - L > 16) {
          // ids of a row are spread over [0, num_nodes): x is expected near L + x * n / num_nodes
          slope = (float)(H - L) * a.inv_num_nodes;
          p = min(max(L + (int64_t)((float)x * slope), L), H - 1);
          pos = p;
          state = kProbe1;
        } else {
          state = kBinary;
        }
        break;
      case kProbe1: {
        if (v == x) { resolve(true); break; }
        if (v < x) L = p + 1; else H = p;
        const int64_t p2 = min(max(p + (int64_t)((float)(x - v) * slope), prev_lo), prev_hi - 1);
        right = v < x;
        step = 1;
        if (p2 != p) { p = p2; pos = p2; state = kProbe2; } else state = kGallop;
        break;
      }
      case kProbe2:
        if (v == x) { resolve(true); break; }
        if (v < x) L = max(L, p + 1); else H = min(H, p);
        right = v < x;
        step = 1;
        state = kGallop;
        break;
      case kGallop:                         // doubling search away from the last probe towards x
        if (v == x) { resolve(true); break; }
        if (right) { if (v < x) { L = pos + 1; step <<= 1; } else { H = pos; state = kBinary; } }
        else       { if (v > x) { H = pos; step <<= 1; } else { L = pos + 1; state = kBinary; } }
        break;
      case kBinary:
        if (v == x) { resolve(true); break; }
        if (v < x) L = pos + 1; else H = pos;
        break;
      default:
        break;
    }
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
  a.num_walks = num_walks;
  a.id_base = id_base;
  a.seed = seed;
  a.walk_len = walk_len;
  a.inv_p = 1.0f / p;
  a.inv_q = 1.0f / q;
  a.max_bias = fmaxf(a.inv_p, fmaxf(1.0f, a.inv_q));
  a.inv_num_nodes = g->num_nodes > 0 ? 1.0f / (float)g->num_nodes : 0.0f;
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
