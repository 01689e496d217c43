// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include "fcp.h"

namespace fcp {

// Records a thread-local error message and returns `code`.
int fail(int code, const char* fmt, ...);
void clear_error();

#define FCP_HIP_CHECK(expr)                                                          \
  do {                                                                               \
    hipError_t e__ = (expr);                                                         \
    if (e__ != hipSuccess)                                                           \
      return ::fcp::fail(FCP_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

// A kernel that uses more than 64 KB of dynamic LDS needs its limit raised once per device; `done` keeps one bit
// per device (devices past 63 raise it on every call).  Safe to call from several threads.
inline int raise_lds_limit(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return FCP_OK;
  FCP_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  done.fetch_or(bit, std::memory_order_release);
  return FCP_OK;
}

// ---- device-side schedule kept at the start of the caller's scratch buffer ----------
// Both attention kernels are persistent: blocks pull (tile, head) units from counters
// until the list is exhausted.  There is one counter per XCD so that the blocks of one
// XCD (blockIdx % 8) walk the heads of the same KV heads and share K/V in that XCD's L2.
constexpr int kNumXcd = 8;
struct SchedHeader {
  int32_t n_tiles;              // tiles in the list (sorted by decreasing cost)
  int32_t n_rejected;           // work items that failed validation
  int32_t max_cost;
  int32_t pad0;
  int32_t counter[kNumXcd];     // next unit per XCD (or counter[0] alone)
  int32_t pad1[4];
};                               // 64 bytes
static_assert(sizeof(SchedHeader) == 64, "header size");

// One schedulable tile, fully resolved by the scheduler so that an attention kernel needs a
// single 64-byte read per unit (no dependent loads of work item and cu_seqlens).
struct QTile {                   // a block of query rows of one work item (forward, dQ)
  int32_t q_row0;                // local row of the first query row (q_local_off + offset)
  int32_t q_pos0;                // its position in the sequence
  int32_t rows;                  // rows in the block
  int32_t step;                  // partial slot
  int32_t kv_row0[2];            // pool row of the first key of each segment
  int32_t k_pos0[2];             // its position in the sequence
  int32_t vis[2];                // keys of the segment that the block's last row sees (0 = none)
  int32_t flags;                 // kFlag* of the work item
  int32_t pad[5];
};
struct KTile {                   // a block of keys of one segment of one work item (dK/dV)
  int32_t kv_row0;               // pool row of the first key
  int32_t k_pos0;                // its position in the sequence
  int32_t n_keys;                // keys in the block that some row of the item sees
  int32_t q_local_off, q_seq_start, q_len;   // the item's query rows
  int32_t flags;                 // kFlagSeg0Exclusive set iff no other item touches these keys
  // Per group of 32 keys: the sequence position of the first query that sees the group's first key and of the
  // first query that sees its last key (of the tile's n_keys), both capped at the item's last row.  With the
  // causal mask these are the two keys' own positions; with full-attention spans the start of the key's span.
  int32_t from_first[4], from_last[4];
  int32_t pad;
};
static_assert(sizeof(QTile) == 64 && sizeof(KTile) == 64, "tile records are 16 words");
struct Tile { int32_t w[16]; };  // storage type of the list

constexpr int kFwdBM = 256;      // query rows per forward unit
constexpr int kFwdBN = 64;       // keys per forward inner step
constexpr int kDqBM = 128;       // query rows per dQ unit (two heads of a KV head), twice that for a single head
constexpr int kDqBN = 32;        // keys per dQ inner step
constexpr int kBwdBN = 128;      // keys per dK/dV unit
constexpr int kBwdBM = 32;       // query rows per dK/dV inner step
constexpr int kMinQTile = 128;   // smallest query tile of any kernel (sizes the tile lists)

// Longest key segment of a work item the kernels take.  Byte offsets into a segment travel in 32-bit scalar
// offsets of buffer instructions, and the fills run a few tiles past a segment's end (those land outside the
// resource's range and read as zero): with a segment below 2^30 bytes the offsets stay far from 2^31.
inline int32_t max_segment_keys(int64_t kv_row_bytes) { return (int32_t)(((int64_t)1 << 30) / kv_row_bytes); }

// Upper bounds on the number of tiles of a valid plan (anything beyond is dropped and
// counted as rejected).  Query tiles: every (row, slot) belongs to at most one item, and over
// a rank's items the query chunks of a sequence add up to at most its length.  Key tiles:
// over a rank's items the key segments of a sequence add up to at most twice its length.
int64_t q_tile_cap(int32_t tq, int32_t tkv, int64_t n_work, int32_t n_parts);
int64_t kv_tile_cap(int32_t tkv, int64_t n_work);

// One schedule region: SchedHeader | item offsets int32[n_work+1] | item flags int32[n_work]
// | Tile[cap]; every part padded to 64 bytes, the region to 256.
constexpr int32_t kFlagQExclusive = 1;    // no other item of the launch covers these query rows
constexpr int32_t kFlagSeg0Exclusive = 2; // no other item's key segment overlaps segment 0 / 1
constexpr int32_t kFlagSeg1Exclusive = 4;
inline size_t pad_to(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t sched_item_off_bytes(int64_t n_work) { return pad_to((size_t)(n_work + 1) * sizeof(int32_t), 64); }
inline size_t sched_flags_bytes(int64_t n_work) { return pad_to((size_t)(n_work > 0 ? n_work : 1) * sizeof(int32_t), 64); }
inline size_t sched_region_bytes(int64_t n_work, int64_t cap) {
  return pad_to(sizeof(SchedHeader) + sched_item_off_bytes(n_work) + sched_flags_bytes(n_work) +
                (size_t)cap * sizeof(Tile), 256);
}
inline const SchedHeader* sched_header(const void* region) { return static_cast<const SchedHeader*>(region); }
inline const int32_t* sched_flags(const void* region, int64_t n_work) {
  return reinterpret_cast<const int32_t*>(static_cast<const char*>(region) + sizeof(SchedHeader) +
                                          sched_item_off_bytes(n_work));
}
inline const Tile* sched_tiles(const void* region, int64_t n_work) {
  return reinterpret_cast<const Tile*>(static_cast<const char*>(region) + sizeof(SchedHeader) +
                                       sched_item_off_bytes(n_work) + sched_flags_bytes(n_work));
}

static_assert(kBwdBN == 4 * 32, "KTile keeps four key groups");

struct RowStates;   // direct modes, see below

// Builds one tile list in `region` (tiles of `tile` keys if `key_tiles`, else of `tile` query rows;
// `inner` is the block size of the other dimension used for the cost; kv_row_bytes = hkv*D*2 bounds
// the segment length so that byte offsets inside a segment fit 31 bits) and, when
// lse_fill is given, fills it with -inf.
// q_limit [tq] / k_from [tkv] (device, or NULL for the causal mask): last key position a local query row
// sees / first query position that sees a pool key.
int launch_schedule(bool key_tiles, int32_t tile, int32_t inner, int64_t kv_row_bytes,
                    const int32_t* q_limit, const int32_t* k_from,
                    const fcp_work_desc* work, int64_t n_work,
                    const int32_t* cu_seqlens_kv, int32_t n_seqs, int32_t tq, int32_t tkv,
                    int32_t n_parts, int64_t tile_cap, void* region, float* lse_fill,
                    int64_t lse_fill_n, hipStream_t stream, const RowStates* states = nullptr);

// Everything that precedes the backward's attention kernels in one launch: both tile lists (key tiles of kBwdBN
// keys in region_kv, query tiles of dq_tile rows in region_q) and the row statistics (stats: two planes of n_stats
// floats, -LSE log2 e and -delta).
int launch_schedule_bwd(int64_t kv_row_bytes, const int32_t* q_limit, const int32_t* k_from,
                        const fcp_work_desc* work, int64_t n_work, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                        int32_t tq, int32_t tkv, int64_t cap_kv, void* region_kv, int32_t dq_tile, int64_t cap_q, void* region_q,
                        const float* lse, const float* delta, int64_t n_stats, float* stats, hipStream_t stream,
                        const RowStates* states = nullptr);

// Direct modes: one state byte per query row and (backward: kv_state not NULL) per pool key: 0 untouched, 1 several
// work items contribute (backward: accumulated in fp32, the accumulator row is cleared when the accumulators are
// given; forward: partial results, merged afterwards), 2 written directly as bf16 by the unit that owns it.
// n_parts / check_step: the validity rules of the list the states go with.  The scheduling launches below compute
// them on additional blocks when `states` is given; launch_row_states() is the same work as a launch of its own.
struct RowStates {
  uint8_t* q_state;
  uint8_t* kv_state;
  float* dq_acc;
  float* dk_acc;
  float* dv_acc;
  int32_t q_row_elems, kv_row_elems;
  int32_t n_parts;
  bool check_step;
};
int launch_row_states(int64_t kv_row_bytes, const RowStates& rs, const int32_t* q_limit, const int32_t* k_from,
                      const fcp_work_desc* work, int64_t n_work, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                      int32_t tq, int32_t tkv, hipStream_t stream);

// Where the row states live in the backward's scratch buffer (after the two lists and the statistics planes).
inline uint8_t* bwd_q_state(void* scratch, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq) {
  return static_cast<uint8_t*>(scratch) + sched_region_bytes(n_work, kv_tile_cap(tkv, n_work)) +
         sched_region_bytes(n_work, q_tile_cap(tq, tkv, n_work, 1 << 20)) + pad_to((size_t)hq * (size_t)tq * 8, 256);
}
inline uint8_t* bwd_kv_state(void* scratch, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq) {
  return bwd_q_state(scratch, n_work, tq, tkv, hq) + pad_to((size_t)tq, 256);
}

// The forward's row states follow its tile list in its scratch buffer.
inline uint8_t* fwd_q_state(void* scratch, int64_t n_work, int32_t tq, int32_t tkv, int32_t n_parts) {
  return static_cast<uint8_t*>(scratch) + sched_region_bytes(n_work, q_tile_cap(tq, tkv, n_work, n_parts));
}

}  // namespace fcp
