// Device-side tile scheduler for the attention kernels.
//
// The paper's motivation (Sec. 4.1) is that heterogeneous lengths leave some compute units
// as stragglers; inside one rank the same holds for tiles: a query block at the end of a long
// chunk has hundreds of key blocks, one from a short sequence has one.  This kernel turns the
// rank's work items (device memory) into a list of tiles sorted by DECREASING cost, which the
// persistent attention kernels pull from shared counters (longest-first list scheduling).
// Fully masked key blocks never enter the cost or the kernels' loops.
//
// It also validates every work item against the extents the caller passed, so that no
// attention kernel can be steered out of bounds by a bad descriptor: a rejected item gets
// no tiles and is counted in the header.
#include "fcp_internal.h"

namespace fcp {

namespace {

constexpr int kSchedThreads = 1024;
constexpr int kBuckets = 2048;
constexpr int kMaxExclusiveScan = 1024;   // beyond this many items the all-pairs overlap scan is skipped

struct ItemInfo {
  bool ok;
  int32_t n_tiles;     // tiles this item contributes
  int32_t nt0;         // backward: tiles of segment 0
  int32_t max_cost;
};

__device__ inline int32_t ceil_div(int32_t a, int32_t b) { return (a + b - 1) / b; }

__device__ inline bool item_valid(const fcp_work_desc& w, const int32_t* cu, int32_t n_seqs,
                                  int32_t tq, int32_t tkv, int32_t n_parts, bool check_step, int32_t max_seg_keys) {
  if (w.seq < 0 || w.seq >= n_seqs) return false;
  if (check_step && (w.step < 0 || w.step >= n_parts)) return false;
  if (w.q_len < 1 || w.q_local_off < 0 || w.q_seq_start < 0) return false;
  if ((int64_t)w.q_local_off + w.q_len > (int64_t)tq) return false;
  if ((int64_t)w.q_seq_start + w.q_len > (int64_t)(1 << 30)) return false;
  if (w.n_seg < 1 || w.n_seg > 2) return false;
  const int64_t s0 = cu[w.seq], s1 = cu[w.seq + 1];
  if (s0 < 0 || s1 < s0 || s1 > (int64_t)tkv) return false;
  for (int s = 0; s < w.n_seg; ++s) {
    if (w.k_seq_start[s] < 0 || w.k_len[s] < 1 || w.k_len[s] > max_seg_keys) return false;
    if (s0 + (int64_t)w.k_seq_start[s] + w.k_len[s] > s1) return false;
  }
  return true;
}

// The mask in the form every kernel uses: row i sees the keys at positions 0 .. limit(i), a key is seen by the
// rows from position from(key) on; both grow with the position.  Causal: limit = the row's own position,
// from = the key's own position; with full-attention spans the tables the caller passed.
struct MaskTables {
  const int32_t* q_limit;   // [tq] by local query row, or NULL
  const int32_t* k_from;    // [tkv] by pool row, or NULL
  __device__ int64_t limit(const fcp_work_desc& w, int32_t row) const {
    return q_limit ? (int64_t)q_limit[w.q_local_off + row] : (int64_t)w.q_seq_start + row;
  }
  __device__ int64_t from(const fcp_work_desc& w, const int32_t* cu, int64_t k_pos) const {
    return k_from ? (int64_t)k_from[cu[w.seq] + k_pos] : k_pos;
  }
};

// keys of segment s that row `last_row` of the item (hence any row up to it) can see
__device__ inline int32_t visible_len(const MaskTables& m, const fcp_work_desc& w, int s, int32_t last_row) {
  int64_t v = m.limit(w, last_row) - w.k_seq_start[s] + 1;
  if (v < 0) v = 0;
  if (v > w.k_len[s]) v = w.k_len[s];
  return (int32_t)v;
}

// query tile qt (of `tile` rows): cost = key blocks (of `inner` keys) its last row sees
__device__ inline int32_t fwd_cost(const MaskTables& m, const fcp_work_desc& w, int32_t qt, int32_t tile, int32_t inner) {
  int32_t last_row = min((qt + 1) * tile, w.q_len) - 1;
  int32_t c = 0;
  for (int s = 0; s < w.n_seg; ++s) c += ceil_div(visible_len(m, w, s, last_row), inner);
  return c;
}

// key tile kt (of `tile` keys) of segment s: cost = query blocks (of `inner` rows) that see its first key
__device__ inline int32_t bwd_cost(const MaskTables& m, const int32_t* cu, const fcp_work_desc& w, int s, int32_t kt,
                                   int32_t tile, int32_t inner) {
  const int64_t first_k_pos = (int64_t)w.k_seq_start[s] + (int64_t)kt * tile;
  int64_t first_row = m.from(w, cu, first_k_pos) - w.q_seq_start;
  if (first_row < 0) first_row = 0;
  const int64_t rows = (int64_t)w.q_len - first_row;
  return rows <= 0 ? 0 : (int32_t)((rows + inner - 1) / inner);
}

__device__ inline ItemInfo item_info(const MaskTables& m, const fcp_work_desc& w, const int32_t* cu, int32_t n_seqs,
                                     int32_t tq, int32_t tkv, int32_t n_parts, bool backward,
                                     bool check_step, int32_t tile, int32_t inner, int32_t max_seg_keys) {
  ItemInfo r{false, 0, 0, 0};
  r.ok = item_valid(w, cu, n_seqs, tq, tkv, n_parts, check_step, max_seg_keys);
  if (!r.ok) return r;
  if (!backward) {
    r.n_tiles = ceil_div(w.q_len, tile);
    r.max_cost = fwd_cost(m, w, r.n_tiles - 1, tile, inner);
  } else {
    r.nt0 = ceil_div(visible_len(m, w, 0, w.q_len - 1), tile);
    int32_t nt1 = w.n_seg > 1 ? ceil_div(visible_len(m, w, 1, w.q_len - 1), tile) : 0;
    r.n_tiles = r.nt0 + nt1;
    r.max_cost = ceil_div(w.q_len, inner);
  }
  return r;
}

// Exclusive block scan of one value per thread; returns the exclusive prefix and sets
// `total` (same for every thread).  `s_wave` holds one slot per wave.
__device__ inline int32_t block_exclusive_scan(int32_t v, int32_t* s_wave, int32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int32_t inc = v;
  for (int off = 1; off < 64; off <<= 1) {
    int32_t t = __shfl_up(inc, off, 64);
    if (lane >= off) inc += t;
  }
  __syncthreads();
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int32_t base = 0, tot = 0;
  for (int w = 0; w < kSchedThreads / 64; ++w) {
    const int32_t x = s_wave[w];
    if (w < wave) base += x;
    tot += x;
  }
  total = tot;
  return base + inc - v;
}

// Exclusivity flags: an item whose query rows (key segments) no other valid item of this launch touches lets the
// backward kernels add to dQ (dK/dV) without atomics, or write the final result directly.  The items' ranges are
// staged in LDS (seq, -1 = invalid; q range; two key ranges) so that the all-pairs scan does not wait on global memory.
__device__ inline void stage_item(int32_t (&r)[7], const fcp_work_desc& a, bool ok) {
  r[0] = ok ? a.seq : -1;
  r[1] = a.q_local_off;
  r[2] = a.q_local_off + a.q_len;
  r[3] = a.k_seq_start[0];
  r[4] = a.k_seq_start[0] + a.k_len[0];
  r[5] = a.n_seg > 1 ? a.k_seq_start[1] : 0;
  r[6] = a.n_seg > 1 ? a.k_seq_start[1] + a.k_len[1] : 0;   // empty range when absent
}
// Flags of all items at once (n_work <= kMaxExclusiveScan), by sorting instead of comparing all pairs: intervals sorted by
// their start overlap an earlier one iff the largest end so far exceeds their start, and a later one iff the next start
// lies before their end.  Query rows: one set over all valid items.  Key segments: one set of up to two segments per
// item, ordered by (sequence, start); only segments of the same sequence can overlap, and an item's own two segments
// count like anybody else's.  The sequence enters the sort key with its low 21 bits: two sequences that collide there
// are treated as one, which can only clear a flag that could have been set (the safe side).
// `key`: LDS work area of 2 * kMaxExclusiveScan entries; `fl`: LDS, one word per item, written here.
__device__ inline void bitonic_sort(uint64_t* key, int32_t n_pow2) {
  // A list written in row order (the usual case: items by sequence, chunks by position) is sorted already: one pass
  // over the neighbours finds that out, and the log^2 rounds of exchanges and block barriers are skipped.
  int ordered = 1;
  for (int32_t t = threadIdx.x; t + 1 < n_pow2; t += kSchedThreads) ordered &= key[t] <= key[t + 1];
  if (__syncthreads_and(ordered)) return;
  for (int32_t k = 2; k <= n_pow2; k <<= 1)
    for (int32_t j = k >> 1; j > 0; j >>= 1) {
      for (int32_t t = threadIdx.x; t < n_pow2 / 2; t += kSchedThreads) {
        const int32_t i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), l = i | j;
        const uint64_t a = key[i], b = key[l];
        if ((a > b) == ((i & k) == 0)) { key[i] = b; key[l] = a; }
      }
      __syncthreads();
    }
}

// Inclusive running maximum over the block's values in thread order (two per thread: v0 then v1).  `s_wmax`: 16 slots.
__device__ inline void block_running_max(uint64_t v0, uint64_t v1, uint64_t* s_wmax, uint64_t& before0, uint64_t& before1) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t inc = v0 > v1 ? v0 : v1;
  for (int off = 1; off < 64; off <<= 1) {
    const uint64_t o = __shfl_up(inc, off, 64);
    if (lane >= off && o > inc) inc = o;
  }
  __syncthreads();
  if (lane == 63) s_wmax[wave] = inc;
  __syncthreads();
  uint64_t base = 0;
  for (int w = 0; w < wave; ++w) base = s_wmax[w] > base ? s_wmax[w] : base;
  uint64_t prev = __shfl_up(inc, 1, 64);        // maximum up to and including the thread before, inside the wave
  if (lane == 0) prev = 0;
  before0 = prev > base ? prev : base;          // maximum of everything before v0
  before1 = before0 > v0 ? before0 : v0;        // ... before v1
}

constexpr int kSmallList = 64;   // up to this many items the flags come from a comparison of all pairs

__device__ inline void exclusive_flags_all(const int32_t (*rng)[7], int32_t n_work, uint64_t* key, uint64_t* s_wmax, int32_t* fl) {
  const int tid = threadIdx.x;
  constexpr uint64_t kNone = ~(uint64_t)0;
  for (int32_t i = tid; i < n_work; i += kSchedThreads)
    fl[i] = rng[i][0] < 0 ? 0 : (kFlagQExclusive | kFlagSeg0Exclusive | kFlagSeg1Exclusive);
  if (n_work <= kSmallList) {
    // Short lists (a packed micro-batch of a few dozen sequences): all pairs of segment slots, 16 or fewer per thread -
    // the two sorts below are 36 or more rounds of LDS traffic and block barriers, 10 us where this takes 1.  The same
    // rules: empty segments and invalid items take no part, sequences compare by their low 21 bits, an item's own
    // other segment counts, query rows are compared once per pair of items.
    __syncthreads();
    const int32_t m = 2 * n_work;
    for (int32_t idx = tid; idx < m * m; idx += kSchedThreads) {
      const int32_t a = idx / m, b = idx - a * m;
      if (a == b) continue;
      const int32_t ia = a >> 1, sa = a & 1, ib = b >> 1, sb = b & 1;
      if (rng[ia][0] < 0 || rng[ib][0] < 0) continue;
      const int32_t a0 = rng[ia][3 + 2 * sa], a1 = rng[ia][4 + 2 * sa], b0 = rng[ib][3 + 2 * sb], b1 = rng[ib][4 + 2 * sb];
      if (a1 > a0 && b1 > b0 && ((rng[ia][0] ^ rng[ib][0]) & 0x1FFFFF) == 0 && a0 < b1 && b0 < a1)
        atomicAnd(&fl[ia], ~(sa ? kFlagSeg1Exclusive : kFlagSeg0Exclusive));
      if (sa == 0 && sb == 0 && rng[ia][1] < rng[ib][2] && rng[ib][1] < rng[ia][2]) atomicAnd(&fl[ia], ~kFlagQExclusive);
    }
    __syncthreads();
    return;
  }
  // ---- query rows: key = start << 11 | item
  int32_t np = 2;
  while (np < n_work) np <<= 1;
  for (int32_t i = tid; i < np; i += kSchedThreads)
    key[i] = (i < n_work && rng[i][0] >= 0) ? ((uint64_t)(uint32_t)rng[i][1] << 11) | (uint64_t)i : kNone;
  __syncthreads();
  bitonic_sort(key, np);
  {
    // one element per thread (np <= kSchedThreads): value of the running maximum = end
    const uint64_t k0 = tid < np ? key[tid] : kNone;
    const bool live = k0 != kNone;
    const int32_t item = live ? (int32_t)(k0 & 2047) : 0;
    const uint64_t end = live ? (uint64_t)(uint32_t)rng[item][2] : 0;
    uint64_t before, unused;
    block_running_max(end, 0, s_wmax, before, unused);
    if (live) {
      const uint64_t start = k0 >> 11;
      const uint64_t nxt = tid + 1 < np ? key[tid + 1] : kNone;
      const bool hit = before > start || (nxt != kNone && (nxt >> 11) < end);
      if (hit) atomicAnd(&fl[item], ~kFlagQExclusive);
    }
  }
  __syncthreads();
  // ---- key segments: key = seq (21 bits) << 43 | start (31 bits) << 12 | slot (item * 2 + segment)
  int32_t np2 = 2;
  while (np2 < 2 * n_work) np2 <<= 1;
  for (int32_t sl = tid; sl < np2; sl += kSchedThreads) {
    const int32_t i = sl >> 1, sg = sl & 1;
    uint64_t k = kNone;
    if (i < n_work && rng[i][0] >= 0) {
      const int32_t a = rng[i][3 + 2 * sg], b = rng[i][4 + 2 * sg];
      if (b > a) k = ((uint64_t)(rng[i][0] & 0x1FFFFF) << 43) | ((uint64_t)(uint32_t)a << 12) | (uint64_t)sl;
    }
    key[sl] = k;
  }
  __syncthreads();
  bitonic_sort(key, np2);
  {
    // two consecutive elements per thread; value of the running maximum = seq << 32 | end
    auto unpack = [&](uint64_t k, uint64_t& val, uint64_t& seqm, uint64_t& start, int32_t& slot) {
      slot = (int32_t)(k & 4095);
      start = (k >> 12) & 0x7FFFFFFFu;
      seqm = k >> 43;
      val = (seqm << 32) | (uint64_t)(uint32_t)rng[slot >> 1][4 + 2 * (slot & 1)];
    };
    const int32_t p0 = 2 * tid, p1 = 2 * tid + 1;
    const uint64_t k0 = p0 < np2 ? key[p0] : kNone, k1 = p1 < np2 ? key[p1] : kNone;
    uint64_t v0 = 0, v1 = 0, q0 = 0, q1 = 0, st0 = 0, st1 = 0;
    int32_t sl0 = 0, sl1 = 0;
    if (k0 != kNone) unpack(k0, v0, q0, st0, sl0);
    if (k1 != kNone) unpack(k1, v1, q1, st1, sl1);
    uint64_t b0, b1;
    block_running_max(v0, v1, s_wmax, b0, b1);
    const uint64_t k2 = p1 + 1 < np2 ? key[p1 + 1] : kNone;
    auto test = [&](uint64_t k, uint64_t val, uint64_t seqm, uint64_t start, int32_t slot, uint64_t before, uint64_t nxt) {
      if (k == kNone) return;
      bool hit = (before >> 32) == seqm && (before & 0xFFFFFFFFu) > start;            // an earlier segment of the sequence ends after this start
      if (nxt != kNone && (nxt >> 43) == seqm && ((nxt >> 12) & 0x7FFFFFFFu) < (val & 0xFFFFFFFFu)) hit = true;   // the next one starts before this end
      if (hit) atomicAnd(&fl[slot >> 1], ~((slot & 1) ? kFlagSeg1Exclusive : kFlagSeg0Exclusive));
    };
    test(k0, v0, q0, st0, sl0, b0, k1);
    test(k1, v1, q1, st1, sl1, b1, k2);
  }
  __syncthreads();
}

// LDS shared between the flags' sort (first) and the list builder's histogram and offsets (afterwards).
struct SortArea {
  union {
    uint64_t key[2 * kMaxExclusiveScan];
    struct { int32_t hist[kBuckets]; int32_t off[kMaxExclusiveScan + 1]; } later;
  };
  uint64_t wmax[kSchedThreads / 64];
};

// One tile list, built by one block.
__device__ void build_list(
    int backward, int check_step, int32_t tile, int32_t inner, int32_t max_seg_keys, const MaskTables m,
    const fcp_work_desc* __restrict__ work, int32_t n_work,
    const int32_t* __restrict__ cu, int32_t n_seqs, int32_t tq, int32_t tkv, int32_t n_parts,
    int32_t tile_cap, SchedHeader* hdr, int32_t* item_off, int32_t* item_flags, Tile* tiles,
    int32_t (*s_rng)[7],                 // LDS, kMaxExclusiveScan rows: seq (-1 = invalid), q range, two key ranges
    SortArea* area, int32_t* s_fl) {     // LDS: sort keys (later the histogram and the offsets), one flag word per item
  __shared__ int32_t s_wave[kSchedThreads / 64];
  __shared__ int32_t s_max, s_rej, s_carry;
  int32_t* const s_hist = area->later.hist;
  int32_t* const s_off = area->later.off;          // copy of item_off for short work lists: the tile decode below
  const bool off_in_lds = n_work <= kMaxExclusiveScan;   // searches it, and a search in global memory is a chain of misses
  const int tid = threadIdx.x;
  // The exclusivity flags first: their sort keys share LDS with the histogram and the offsets.
  if (n_work <= kMaxExclusiveScan) {
    for (int32_t i = tid; i < n_work; i += kSchedThreads) {
      const fcp_work_desc a = work[i];
      stage_item(s_rng[i], a, item_valid(a, cu, n_seqs, tq, tkv, n_parts, check_step != 0, max_seg_keys));
    }
    __syncthreads();
    exclusive_flags_all(s_rng, n_work, area->key, area->wmax, s_fl);
    for (int32_t i = tid; i < n_work; i += kSchedThreads) item_flags[i] = s_fl[i];
  } else {
    for (int32_t i = tid; i < n_work; i += kSchedThreads) item_flags[i] = 0;
  }
  __syncthreads();
  if (tid == 0) { s_max = 0; s_rej = 0; s_carry = 0; }
  for (int b = tid; b < kBuckets; b += kSchedThreads) s_hist[b] = 0;
  __syncthreads();

  // Pass 1: validate, count tiles per item, exclusive offsets into item_off[0..n_work].
  for (int32_t base = 0; base < n_work; base += kSchedThreads) {
    const int32_t i = base + tid;
    int32_t cnt = 0;
    if (i < n_work) {
      const fcp_work_desc w = work[i];
      const ItemInfo info = item_info(m, w, cu, n_seqs, tq, tkv, n_parts, backward != 0, check_step != 0, tile, inner, max_seg_keys);
      if (!info.ok) atomicAdd(&s_rej, 1);
      cnt = info.n_tiles;
      if (info.max_cost > 0) atomicMax(&s_max, info.max_cost);
    }
    int32_t total;
    const int32_t ex = block_exclusive_scan(cnt, s_wave, total);
    const int32_t carry = s_carry;
    if (i < n_work) {
      item_off[i] = carry + ex;
      if (off_in_lds) s_off[i] = carry + ex;
    }
    __syncthreads();
    if (tid == 0) s_carry = carry + total;
    __syncthreads();
  }
  const int32_t total_tiles = s_carry;
  const int32_t n_tiles = min(total_tiles, tile_cap);
  if (tid == 0) {
    item_off[n_work] = total_tiles;
    if (total_tiles > tile_cap) atomicAdd(&s_rej, total_tiles - tile_cap);
  }
  int shift = 0;
  while ((s_max >> shift) >= kBuckets) ++shift;
  __syncthreads();

  // Pass 2 and 3 share the decode of a flat tile number into its resolved record and cost.
  auto decode = [&](int32_t t, Tile& out) -> int32_t {
    int32_t lo = 0, hi = n_work - 1;               // last item with item_off <= t
    while (lo < hi) {
      const int32_t mid = (lo + hi + 1) >> 1;
      if ((off_in_lds ? s_off[mid] : item_off[mid]) <= t) lo = mid; else hi = mid - 1;
    }
    const fcp_work_desc w = work[lo];
    const int32_t local = t - (off_in_lds ? s_off[lo] : item_off[lo]);
    const int32_t row0_kv = cu[w.seq];
    const int32_t fl = off_in_lds ? s_fl[lo] : 0;
    for (int i = 0; i < 16; ++i) out.w[i] = 0;
    if (!backward) {
      QTile* q = reinterpret_cast<QTile*>(&out);
      const int32_t r0 = local * tile;
      q->q_row0 = w.q_local_off + r0;
      q->q_pos0 = w.q_seq_start + r0;
      q->rows = min(tile, w.q_len - r0);
      q->step = w.step;
      for (int sg = 0; sg < 2; ++sg) {
        q->kv_row0[sg] = sg < w.n_seg ? row0_kv + w.k_seq_start[sg] : 0;
        q->k_pos0[sg] = sg < w.n_seg ? w.k_seq_start[sg] : 0;
        q->vis[sg] = sg < w.n_seg ? visible_len(m, w, sg, r0 + q->rows - 1) : 0;
      }
      q->flags = fl;
      return fwd_cost(m, w, local, tile, inner);
    }
    const int32_t nt0 = ceil_div(visible_len(m, w, 0, w.q_len - 1), tile);
    const int sg = local >= nt0 ? 1 : 0;
    const int32_t kt = local - (sg ? nt0 : 0);
    KTile* k = reinterpret_cast<KTile*>(&out);
    k->kv_row0 = row0_kv + w.k_seq_start[sg] + kt * tile;
    k->k_pos0 = w.k_seq_start[sg] + kt * tile;
    k->n_keys = min(tile, visible_len(m, w, sg, w.q_len - 1) - kt * tile);
    const int64_t last_q_pos = (int64_t)w.q_seq_start + w.q_len - 1;
    for (int g = 0; g < 4; ++g) {
      const int32_t first_key = min(32 * g, k->n_keys - 1), last_key = min(32 * g + 31, k->n_keys - 1);
      k->from_first[g] = (int32_t)min(last_q_pos, m.from(w, cu, (int64_t)k->k_pos0 + first_key));
      k->from_last[g] = (int32_t)min(last_q_pos, m.from(w, cu, (int64_t)k->k_pos0 + last_key));
    }
    k->q_local_off = w.q_local_off;
    k->q_seq_start = w.q_seq_start;
    k->q_len = w.q_len;
    k->flags = (fl & (sg ? kFlagSeg1Exclusive : kFlagSeg0Exclusive)) ? kFlagSeg0Exclusive : 0;
    return bwd_cost(m, cu, w, sg, kt, tile, inner);
  };

  // (a thread's first tile and its cost stay in registers for the scatter pass: with up to 1024 tiles, all of them)
  Tile first_tile;
  int32_t first_cost = 0;
  for (int32_t t = tid; t < n_tiles; t += kSchedThreads) {
    Tile tl;
    const int32_t c = decode(t, tl);
    if (t == tid) { first_tile = tl; first_cost = c; }
    atomicAdd(&s_hist[min(c >> shift, kBuckets - 1)], 1);
  }
  __syncthreads();
  // Descending-cost start offset of every bucket: scan the histogram from the top.
  {
    static_assert(kBuckets == 2 * kSchedThreads, "two buckets per thread");
    const int b_hi = kBuckets - 1 - 2 * tid, b_lo = b_hi - 1;
    const int32_t h_hi = s_hist[b_hi], h_lo = s_hist[b_lo];
    int32_t total;
    const int32_t ex = block_exclusive_scan(h_hi + h_lo, s_wave, total);
    __syncthreads();
    s_hist[b_hi] = ex;
    s_hist[b_lo] = ex + h_hi;
  }
  __syncthreads();
  for (int32_t t = tid; t < n_tiles; t += kSchedThreads) {
    Tile tl;
    int32_t c;
    if (t == tid) { tl = first_tile; c = first_cost; }
    else c = decode(t, tl);
    const int32_t pos = atomicAdd(&s_hist[min(c >> shift, kBuckets - 1)], 1);
    tiles[pos] = tl;
  }
  if (tid == 0) {
    hdr->n_tiles = n_tiles;
    hdr->n_rejected = s_rej;
    hdr->max_cost = s_max;
    hdr->pad0 = 0;
    for (int c = 0; c < 4; ++c) hdr->pad1[c] = 0;
    for (int c = 0; c < kNumXcd; ++c) hdr->counter[c] = 0;
  }
}

// Direct mode of the backward: where does the result of every query row / pool key come from?  State 0: no unit of
// this launch touches it (the result is zero); 1: it is accumulated in fp32 (several units, atomics) and converted
// afterwards - its accumulator row is cleared here; 2: one unit owns it and writes the final bf16 row itself.  The
// states follow the same exclusivity flags the kernels act on.  One lane per row, 64-row batches dealt out to the blocks in turn.
struct RowStateJob {
  uint8_t* q_state;        // NULL: no row states in this launch
  uint8_t* kv_state;       // NULL: query rows only (forward)
  float* dq_acc;           // accumulators whose state-1 rows are cleared, or NULL
  float* dk_acc;
  float* dv_acc;
  int32_t q_row_elems, kv_row_elems;
  int32_t n_parts, check_step;   // the validity rules of the list the states go with
};
// The blocks `first` .. `first + count - 1` of the launch share the rows; LDS arrays come from the kernel.
__device__ void row_states(
    int first, int count, const RowStateJob& job, int32_t max_seg_keys, const MaskTables& m,
    const fcp_work_desc* __restrict__ work, int32_t n_work, const int32_t* __restrict__ cu, int32_t n_seqs, int32_t tq,
    int32_t tkv, int32_t (*s_rng)[7], int32_t (*s_vis)[2], int32_t* s_fl, SortArea* area) {
  uint8_t* __restrict__ q_state = job.q_state;
  uint8_t* __restrict__ kv_state = job.kv_state;
  float* __restrict__ dq_acc = job.dq_acc;
  float* __restrict__ dk_acc = job.dk_acc;
  float* __restrict__ dv_acc = job.dv_acc;
  const int32_t q_row_elems = job.q_row_elems, kv_row_elems = job.kv_row_elems;
  const int32_t n_kv_rows = kv_state ? tkv : 0;
  const int tid = threadIdx.x, lane = tid & 63;
  for (int32_t i = tid; i < n_work; i += kSchedThreads) {
    const fcp_work_desc a = work[i];
    const bool ok = item_valid(a, cu, n_seqs, tq, tkv, job.n_parts, job.check_step != 0, max_seg_keys);
    stage_item(s_rng[i], a, ok);
    s_vis[i][0] = ok ? visible_len(m, a, 0, a.q_len - 1) : 0;
    s_vis[i][1] = ok && a.n_seg > 1 ? visible_len(m, a, 1, a.q_len - 1) : 0;
  }
  __syncthreads();
  exclusive_flags_all(s_rng, n_work, area->key, area->wmax, s_fl);
  // The key ranges as pool rows [first, end of the visible part): a pool row then needs no search for its sequence
  // (a binary search of cu_seqlens per row, ten dependent trips to global memory, was most of this pass).  A rejected
  // item gets empty ranges, so the passes over the list below carry no test of validity.
  for (int32_t i = tid; i < n_work; i += kSchedThreads) {
    if (s_rng[i][0] < 0) {
      for (int c = 1; c < 7; ++c) s_rng[i][c] = 0;
    } else if (n_kv_rows > 0) {
      const int32_t base = cu[s_rng[i][0]];
      s_rng[i][3] += base;
      s_rng[i][4] = s_rng[i][3] + s_vis[i][0];
      s_rng[i][5] += base;
      s_rng[i][6] = s_rng[i][5] + s_vis[i][1];
    }
  }
  __syncthreads();

  // Rows are taken in batches of 64, one LANE per row.  Batch f belongs to block f mod count, so every block's batches
  // are spread evenly over all rows: any run of rows that must be cleared is shared by all blocks, and a block still
  // meets only the items that reach into one of its batches (for many short sequences a small part of the list),
  // which it picks first.  A wave then walks the picked items for its 64 rows (all lanes read the same item, an LDS
  // broadcast; nothing is exchanged between lanes).  The rows that are accumulated into go to a list in LDS, and the
  // block's 16 waves clear them in turn.  (Every row against every item, one wave per row and a search of cu_seqlens
  // per pool row, took 0.33 ms for 256 K rows and 1000 items.)
  const int64_t n_rows = (int64_t)tq + n_kv_rows;     // (the forward classifies its query rows only)
  const int64_t n_batches = (n_rows + 63) >> 6;
  const int64_t blk = blockIdx.x - first;
  const int wave = tid >> 6;
  int32_t* s_pick = reinterpret_cast<int32_t*>(area->key);                       // free again once the flags are known
  int64_t* s_clear = reinterpret_cast<int64_t*>(area->key + kMaxExclusiveScan);  // kSchedThreads rows at most
  int32_t* s_cnt = reinterpret_cast<int32_t*>(&area->wmax[0]);                   // [0] items picked, [1] rows to clear
  if (tid == 0) s_cnt[0] = 0;
  __syncthreads();
  {
    // does the range of rows [s, e) meet a batch of this block?  The first batch at or after s / 64 that is ours.
    auto mine = [&](int64_t s0, int64_t e0) {
      if (e0 <= s0) return false;
      const int64_t fs = s0 >> 6;
      int64_t d = (blk - fs) % count;
      if (d < 0) d += count;
      return ((fs + d) << 6) < e0;
    };
    for (int32_t i = tid; i < n_work; i += kSchedThreads) {
      bool hit = mine(s_rng[i][1], s_rng[i][2]);                                 // (a rejected item has empty ranges)
      if (n_kv_rows > 0)
        hit = hit || mine((int64_t)tq + s_rng[i][3], (int64_t)tq + s_rng[i][4]) ||
              mine((int64_t)tq + s_rng[i][5], (int64_t)tq + s_rng[i][6]);
      if (hit) s_pick[atomicAdd(&s_cnt[0], 1)] = i;
    }
  }
  __syncthreads();
  const int32_t n_cand = s_cnt[0];
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  const int64_t per_round = (int64_t)count * (kSchedThreads / 64);
  for (int64_t f0 = 0; f0 < n_batches; f0 += per_round) {    // the same trip count for every wave of the block
    if (tid == 0) s_cnt[1] = 0;
    const int64_t f = f0 + (int64_t)wave * count + blk;
    const int64_t r0 = f << 6, r = r0 + lane;
    const bool live = r < n_rows;
    int32_t cnt = 0, own = 0;            // covering (item, segment) pairs; flags bit of the last one found
    // (no branch inside these loops: the reads of several items are in flight together)
    if (r0 + 63 < tq) {                  // 64 query rows
      const int32_t x = (int32_t)r;
#pragma unroll 4
      for (int32_t c = 0; c < n_cand; ++c) {
        const int32_t j = s_pick[c];
        const bool hit = s_rng[j][1] <= x && x < s_rng[j][2];
        cnt += hit;
        own = hit ? s_fl[j] & kFlagQExclusive : own;
      }
    } else if (r0 < n_rows) {            // pool rows, or the batch with the last query rows and the first pool rows
      const bool is_q = r < tq;
      const int32_t x = (int32_t)(is_q ? r : r - tq);
#pragma unroll 4
      for (int32_t c = 0; c < n_cand; ++c) {
        const int32_t j = s_pick[c];
        const int32_t fj = s_fl[j];
        const bool hq = is_q && s_rng[j][1] <= x && x < s_rng[j][2];
        const bool h0 = !is_q && s_rng[j][3] <= x && x < s_rng[j][4];
        const bool h1 = !is_q && s_rng[j][5] <= x && x < s_rng[j][6];
        cnt += (int)hq + (int)h0 + (int)h1;
        own = hq ? fj & kFlagQExclusive : own;
        own = h0 ? fj & kFlagSeg0Exclusive : own;
        own = h1 ? fj & kFlagSeg1Exclusive : own;
      }
    }
    const int state = cnt == 0 ? 0 : (cnt == 1 && own != 0) ? 2 : 1;
    if (live) {
      if (r < tq) q_state[r] = (uint8_t)state;
      else kv_state[r - tq] = (uint8_t)state;
    }
    __syncthreads();
    const bool clear = live && state == 1 && (r >= tq || dq_acc != nullptr);
    const uint64_t todo = __builtin_amdgcn_ballot_w64(clear);
    if (todo) {
      int32_t base = 0;
      if (lane == 0) base = atomicAdd(&s_cnt[1], __builtin_popcountll(todo));
      base = __builtin_amdgcn_readfirstlane(base);
      const int32_t pos = base + (int32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(todo >> 32),
                                                                     __builtin_amdgcn_mbcnt_lo((uint32_t)todo, 0));
      if (clear) s_clear[pos] = r;
    }
    __syncthreads();
    const int32_t n_clear = s_cnt[1];
    for (int32_t c = wave; c < n_clear; c += kSchedThreads / 64) {
      const int64_t rr = s_clear[c];
      if (rr < tq) {
        float4* row = reinterpret_cast<float4*>(dq_acc + rr * q_row_elems);
        for (int32_t e = lane; e < q_row_elems / 4; e += 64) row[e] = zero;
      } else {
        const int64_t kr = rr - tq;
        float4* rk = reinterpret_cast<float4*>(dk_acc + kr * kv_row_elems);
        float4* rv = reinterpret_cast<float4*>(dv_acc + kr * kv_row_elems);
        for (int32_t e = lane; e < kv_row_elems / 4; e += 64) { rk[e] = zero; rv[e] = zero; }
      }
    }
    __syncthreads();
  }
}

// The row states alone (launches that build no list).
__global__ __launch_bounds__(kSchedThreads) void row_state_kernel(
    const RowStateJob job, int32_t max_seg_keys, const MaskTables m, const fcp_work_desc* __restrict__ work,
    int32_t n_work, const int32_t* __restrict__ cu, int32_t n_seqs, int32_t tq, int32_t tkv) {
  __shared__ int32_t s_rng[kMaxExclusiveScan][7];
  __shared__ int32_t s_vis[kMaxExclusiveScan][2];   // keys of each segment that the item's last row sees
  __shared__ int32_t s_fl[kMaxExclusiveScan];
  __shared__ SortArea s_area;
  row_states(0, gridDim.x, job, max_seg_keys, m, work, n_work, cu, n_seqs, tq, tkv, s_rng, s_vis, s_fl, &s_area);
}

// Forward: block 0 builds the query-tile list, the next `fill_blocks` blocks pre-fill the partial LSE with -inf,
// the blocks after those classify the rows (direct mode).
__global__ __launch_bounds__(kSchedThreads) void sched_kernel(
    int backward, int check_step, int32_t tile, int32_t inner, int32_t max_seg_keys, const MaskTables m,
    const fcp_work_desc* __restrict__ work, int32_t n_work,
    const int32_t* __restrict__ cu, int32_t n_seqs, int32_t tq, int32_t tkv, int32_t n_parts,
    int32_t tile_cap, SchedHeader* hdr, int32_t* item_off, int32_t* item_flags, Tile* tiles,
    float* lse_fill, int64_t lse_fill_n, int fill_blocks, const RowStateJob states) {
  __shared__ int32_t s_rng[kMaxExclusiveScan][7];
  __shared__ int32_t s_vis[kMaxExclusiveScan][2];
  __shared__ int32_t s_fl[kMaxExclusiveScan];
  __shared__ SortArea s_area;
  const int b = blockIdx.x;
  if (b == 0) {
    build_list(backward, check_step, tile, inner, max_seg_keys, m, work, n_work, cu, n_seqs, tq, tkv, n_parts, tile_cap,
               hdr, item_off, item_flags, tiles, s_rng, &s_area, s_fl);
  } else if (b <= fill_blocks) {
    const int64_t stride = (int64_t)fill_blocks * kSchedThreads;
    for (int64_t i = (int64_t)(b - 1) * kSchedThreads + threadIdx.x; i < lse_fill_n; i += stride)
      lse_fill[i] = -INFINITY;
  } else {
    row_states(1 + fill_blocks, gridDim.x - 1 - fill_blocks, states, max_seg_keys, m, work, n_work, cu, n_seqs, tq, tkv,
               s_rng, s_vis, s_fl, &s_area);
  }
}

// Backward: one launch for everything that precedes the two attention kernels.  Block 0 builds the key-tile list
// (dK/dV kernel), block 1 the query-tile list (dQ kernel), the other blocks write the row statistics in the form
// the kernels consume: plane 0 = -LSE log2 e (-inf for a row without keys, so that its probabilities vanish),
// plane 1 = -delta.
struct ListJob {
  int32_t tile, inner, tile_cap;
  SchedHeader* hdr;
  int32_t* item_off;
  int32_t* item_flags;
  Tile* tiles;
};
__global__ __launch_bounds__(kSchedThreads) void sched_bwd_kernel(
    const ListJob kv, const ListJob qt, int32_t max_seg_keys, const MaskTables m,
    const fcp_work_desc* __restrict__ work, int32_t n_work,
    const int32_t* __restrict__ cu, int32_t n_seqs, int32_t tq, int32_t tkv,
    const float* __restrict__ lse, const float* __restrict__ delta, int64_t n_stats, float* __restrict__ stats,
    int stat_blocks, const RowStateJob states) {
  __shared__ int32_t s_rng[kMaxExclusiveScan][7];
  __shared__ int32_t s_vis[kMaxExclusiveScan][2];
  __shared__ int32_t s_fl[kMaxExclusiveScan];
  __shared__ SortArea s_area;
  const int b = blockIdx.x;
  if (b < 2) {
    const ListJob& j = b == 0 ? kv : qt;
    build_list(b == 0 ? 1 : 0, 0, j.tile, j.inner, max_seg_keys, m, work, n_work, cu, n_seqs, tq, tkv, 1,
               j.tile_cap, j.hdr, j.item_off, j.item_flags, j.tiles, s_rng, &s_area, s_fl);
  } else if (b < 2 + stat_blocks) {
    const int64_t stride = (int64_t)stat_blocks * kSchedThreads;
    for (int64_t i = (int64_t)(b - 2) * kSchedThreads + threadIdx.x; i < n_stats; i += stride) {
      const float l = lse[i];
      stats[i] = l == -INFINITY ? -INFINITY : -l * 1.4426950408889634f;
      stats[n_stats + i] = -delta[i];
    }
  } else {   // direct mode: the row states, and the accumulator rows that are accumulated into cleared
    row_states(2 + stat_blocks, gridDim.x - 2 - stat_blocks, states, max_seg_keys, m, work, n_work, cu, n_seqs, tq, tkv,
               s_rng, s_vis, s_fl, &s_area);
  }
}

}  // namespace

constexpr int kRowStateBlocks = 128;
static int row_state_blocks(int32_t tq, int32_t n_kv_rows) {
  int64_t blocks = ((int64_t)tq + n_kv_rows + kSchedThreads / 64 - 1) / (kSchedThreads / 64);
  // Every block stages the whole work list first, so few blocks with several rows per wave.  Measured on the 32K
  // workload (forward / backward scheduling launch): 64 blocks 34 / 81 us, 128 blocks 28 / 50, 256 blocks - / 57,
  // 512 blocks 41 / 58.
  if (blocks > kRowStateBlocks) blocks = kRowStateBlocks;
  return blocks < 1 ? 1 : (int)blocks;
}

static RowStateJob make_job(const RowStates* rs) {
  RowStateJob j{};
  if (rs) {
    j.q_state = rs->q_state; j.kv_state = rs->kv_state;
    j.dq_acc = rs->dq_acc; j.dk_acc = rs->dk_acc; j.dv_acc = rs->dv_acc;
    j.q_row_elems = rs->q_row_elems; j.kv_row_elems = rs->kv_row_elems;
    j.n_parts = rs->n_parts; j.check_step = rs->check_step ? 1 : 0;
  }
  return j;
}

int check_row_states(int64_t n_work) {
  if (n_work > kMaxExclusiveScan)
    return fail(FCP_ERR_UNSUPPORTED, "direct mode: more than %d work items (use the plain entry point)", kMaxExclusiveScan);
  return FCP_OK;
}

int launch_row_states(int64_t kv_row_bytes, const RowStates& rs, const int32_t* q_limit, const int32_t* k_from,
                      const fcp_work_desc* work, int64_t n_work, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                      int32_t tq, int32_t tkv, hipStream_t stream) {
  int rc = check_row_states(n_work);
  if (rc != FCP_OK) return rc;
  hipLaunchKernelGGL(row_state_kernel, dim3((unsigned)row_state_blocks(tq, rs.kv_state ? tkv : 0)), dim3(kSchedThreads), 0,
                     stream, make_job(&rs), max_segment_keys(kv_row_bytes),
                     MaskTables{q_limit, k_from}, work, (int32_t)n_work, cu_seqlens_kv, n_seqs, tq, tkv);
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

int64_t q_tile_cap(int32_t tq, int32_t tkv, int64_t n_work, int32_t n_parts) {
  const int64_t by_slots = (int64_t)n_parts * ((tq + kMinQTile - 1) / kMinQTile);
  const int64_t by_tokens = (int64_t)((tkv + kMinQTile - 1) / kMinQTile);
  return n_work + (by_slots < by_tokens ? by_slots : by_tokens);
}

int64_t kv_tile_cap(int32_t tkv, int64_t n_work) {
  return 2 * n_work + 2 * (int64_t)((tkv + kBwdBN - 1) / kBwdBN);
}

int launch_schedule(bool backward, int32_t tile, int32_t inner, int64_t kv_row_bytes,
                    const int32_t* q_limit, const int32_t* k_from,
                    const fcp_work_desc* work, int64_t n_work,
                    const int32_t* cu_seqlens_kv, int32_t n_seqs, int32_t tq, int32_t tkv,
                    int32_t n_parts, int64_t tile_cap, void* region, float* lse_fill,
                    int64_t lse_fill_n, hipStream_t stream, const RowStates* states) {
  if (states) { const int rcs = check_row_states(n_work); if (rcs != FCP_OK) return rcs; }
  char* base = static_cast<char*>(region);
  SchedHeader* hdr = reinterpret_cast<SchedHeader*>(base);
  int32_t* item_off = reinterpret_cast<int32_t*>(base + sizeof(SchedHeader));
  int32_t* item_flags = const_cast<int32_t*>(sched_flags(region, n_work));
  Tile* tiles = const_cast<Tile*>(sched_tiles(region, n_work));
  int fill_blocks = 0;
  if (lse_fill && lse_fill_n > 0) {
    fill_blocks = (int)((lse_fill_n + kSchedThreads * 4 - 1) / (kSchedThreads * 4));
    if (fill_blocks > 1024) fill_blocks = 1024;
    if (fill_blocks < 1) fill_blocks = 1;
  }
  const int state_blocks = states ? row_state_blocks(tq, states->kv_state ? tkv : 0) : 0;
  hipLaunchKernelGGL(sched_kernel, dim3(1 + fill_blocks + state_blocks), dim3(kSchedThreads), 0, stream,
                     backward ? 1 : 0, lse_fill ? 1 : 0, tile, inner,
                     max_segment_keys(kv_row_bytes), MaskTables{q_limit, k_from}, work, (int32_t)n_work, cu_seqlens_kv, n_seqs, tq, tkv, n_parts,
                     (int32_t)tile_cap, hdr, item_off, item_flags, tiles, lse_fill, lse_fill_n, fill_blocks, make_job(states));
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

int launch_schedule_bwd(int64_t kv_row_bytes, const int32_t* q_limit, const int32_t* k_from,
                        const fcp_work_desc* work, int64_t n_work, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                        int32_t tq, int32_t tkv, int64_t cap_kv, void* region_kv, int32_t dq_tile, int64_t cap_q, void* region_q,
                        const float* lse, const float* delta, int64_t n_stats, float* stats, hipStream_t stream,
                        const RowStates* states) {
  if (states) { const int rcs = check_row_states(n_work); if (rcs != FCP_OK) return rcs; }
  auto job = [&](void* region, int32_t tile, int32_t inner, int64_t cap) {
    ListJob j;
    j.tile = tile; j.inner = inner; j.tile_cap = (int32_t)cap;
    j.hdr = reinterpret_cast<SchedHeader*>(region);
    j.item_off = reinterpret_cast<int32_t*>(static_cast<char*>(region) + sizeof(SchedHeader));
    j.item_flags = const_cast<int32_t*>(sched_flags(region, n_work));
    j.tiles = const_cast<Tile*>(sched_tiles(region, n_work));
    return j;
  };
  int64_t stat_blocks = (n_stats + kSchedThreads * 4 - 1) / (kSchedThreads * 4);
  if (stat_blocks > 1024) stat_blocks = 1024;
  if (stat_blocks < 1) stat_blocks = 1;
  const int state_blocks = states ? row_state_blocks(tq, states->kv_state ? tkv : 0) : 0;
  hipLaunchKernelGGL(sched_bwd_kernel, dim3((unsigned)(2 + stat_blocks + state_blocks)), dim3(kSchedThreads), 0, stream,
                     job(region_kv, kBwdBN, kBwdBM, cap_kv), job(region_q, dq_tile, kDqBN, cap_q),
                     max_segment_keys(kv_row_bytes), MaskTables{q_limit, k_from}, work,
                     (int32_t)n_work, cu_seqlens_kv, n_seqs, tq, tkv, lse, delta, n_stats, stats, (int)stat_blocks,
                     make_job(states));
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

}  // namespace fcp

extern "C" size_t fcp_scratch_bytes(int which, int32_t tq, int32_t tkv, int32_t hq, int32_t hkv,
                                    int32_t head_dim, int64_t n_work, int32_t n_parts) {
  (void)hkv; (void)head_dim;
  if (tq < 0 || tkv < 0 || n_work < 0 || n_parts < 0) return 0;
  if (which == FCP_SCRATCH_BWD)   // key-tile list (dK/dV kernel), query-tile list (dQ kernel), packed row statistics,
                                  // row states
    return fcp::sched_region_bytes(n_work, fcp::kv_tile_cap(tkv, n_work)) +
           fcp::sched_region_bytes(n_work, fcp::q_tile_cap(tq, tkv, n_work, 1 << 20)) +
           fcp::pad_to((size_t)hq * (size_t)tq * 8, 256) +
           fcp::pad_to((size_t)tq, 256) + fcp::pad_to((size_t)tkv, 256);   // + row states of the direct mode
  return fcp::sched_region_bytes(n_work, fcp::q_tile_cap(tq, tkv, n_work, n_parts)) +
         fcp::pad_to((size_t)tq, 256);                                  // + row states of the direct mode
}

extern "C" int fcp_scratch_status(const void* scratch, void* stream, int32_t* n_tiles, int32_t* n_rejected) {
  fcp::clear_error();
  if (!scratch) return fcp::fail(FCP_ERR_INVALID_ARG, "fcp_scratch_status: scratch is NULL");
  fcp::SchedHeader h;
  FCP_HIP_CHECK(hipMemcpyAsync(&h, scratch, sizeof(h), hipMemcpyDeviceToHost, (hipStream_t)stream));
  FCP_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
  if (n_tiles) *n_tiles = h.n_tiles;
  if (n_rejected) *n_rejected = h.n_rejected;
  return FCP_OK;
}
