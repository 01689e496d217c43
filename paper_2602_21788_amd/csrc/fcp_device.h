// Device-side helpers shared by the attention kernels (types, LDS transpose read, lane
// exchange, the persistent-block unit queue).
#pragma once
#include "fcp_internal.h"

namespace fcp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Two 4-row LDS transpose reads (ds_read_b64_tr_b16) -> the 8 k-slots of one MFMA operand.
// Inside a 16-lane block lane i supplies the address of row (i/4), 4 channels at 4*(i%4), and
// receives channel i of rows 0..3: the block's 4 x 16 sub-matrix arrives transposed.
__device__ inline bf16x8 tr_read_8(const unsigned char* p0, int second_off) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0 + second_off));
  return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
}

// Same with the two 4-row reads at unrelated addresses (chunk-permuted tiles).
__device__ inline bf16x8 tr_read_8(const unsigned char* p_lo, const unsigned char* p_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p_lo));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p_hi));
  return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
}

// v_permlane32_swap exchanges the upper half of the first operand with the lower half of the
// second; with both operands = x every lane ends up holding x of lanes l and l^32.
__device__ inline float lane32_partner_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ inline float lane32_partner_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

// Maximum of three as one v_maximum3_f32 (IEEE-754-2019 maximum: no NaN-quieting moves of the inputs,
// which fmaxf brings in IEEE mode).
__device__ inline float max3(float a, float b, float c) {
  return __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c);
}

__device__ inline f32x16 zero16() {
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  return z;
}

// ---- LDS tiles filled by LDS-direct buffer loads ----------------------------------------------
// A wave-wide buffer_load_dwordx4 ... lds puts lane L's 16 bytes at (M0 base) + 16 L (verified on the
// chip; lanes whose address is out of the resource's range write zeros), so a tile row cannot be
// padded.  Bank conflicts are avoided by permuting the 16-byte chunks of a row instead: chunk c of
// tile row r is stored at chunk position c ^ key(r).  Two layouts, both read at the full 256 B/clk:
//   RowTile  rows are read whole as MFMA operands (ds_read_b128, 16 consecutive rows per clock);
//   TrTile   4-row x 64-byte blocks are read with ds_read_b64_tr_b16 (32 lanes per clock).
// s_waitcnt immediate: vmcnt(0) (bits 3:0 and 15:14), expcnt and lgkmcnt left at their maxima.  A
// workgroup barrier does not wait for a wave's outstanding LDS-direct loads by itself.
constexpr int kWaitVm0 = 0x0F70;
#define FCP_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Raw buffer resource: base address, no stride, `bytes` addressable bytes (accesses past them read as
// zero), 32-bit untyped data format.
// The four words are made wave-uniform explicitly (the first lane's values): the LDS-direct loads below take the
// resource in scalar registers, and an operand the compiler cannot prove uniform would otherwise land in vector
// registers, which the instruction does not accept.  `base` and `bytes` must be wave-uniform.
__device__ inline i32x4 buffer_rsrc(const void* base, int bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  const i32x4 r = {__builtin_amdgcn_readfirstlane((int)(uint32_t)a), __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu)),
                   __builtin_amdgcn_readfirstlane(bytes), 0x00020000};
  return r;
}

// LDS byte offset of a __shared__ object (what M0 and the ds instructions take).
__device__ inline uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// One wave-wide LDS-direct load: lane L's 16 bytes from rsrc[voff + soff] land at LDS offset lds + 16 L.
// Written in assembly so that the compiler does not count it among the LDS stores it orders LDS reads
// after (it would make the wave wait for the load just issued before its next LDS read); the caller waits
// with s_waitcnt vmcnt and a barrier before anybody reads the tile.  `lds` and `soff` must be wave-uniform.
// M0 is not used by anything else in these kernels.  The s_nop covers the wait states between the write of M0 and the
// load and, with the s_mov, the five a vector memory instruction needs after a v_readlane that restored one of its
// scalar operands (the compiler pads its own instructions for that hazard, not the inside of an assembly statement).
__device__ inline void lds_fill_b128(i32x4 rsrc, uint32_t lds, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 3\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(__builtin_amdgcn_readfirstlane((int)lds)), "v"(voff), "s"(rsrc), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

template <int D>
struct RowTile {
  static constexpr int CPR = D / 8;        // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;     // rows one wave-wide load instruction fills
  // D = 128: 64 bytes of padding after every 4 rows (one load instruction) + the row's low two bits;
  // D = 64: two rows share a 256-byte bank cycle, so row/2 permutes all 8 chunks.
  __host__ __device__ static constexpr int row_base(int row) { return D == 128 ? row * 256 + (row >> 2) * 64 : row * 128; }
  __host__ __device__ static constexpr int key(int row) { return D == 128 ? (row & 3) : ((row >> 1) & 7); }
  __host__ __device__ static constexpr int bytes(int rows) { return row_base(rows); }
};

template <int D>
struct TrTile {
  static constexpr int CPR = D / 8;
  static constexpr int RPI = 64 / CPR;
  __host__ __device__ static constexpr int row_base(int row) { return row * D * 2; }
  __host__ __device__ static constexpr int key(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
  __host__ __device__ static constexpr int bytes(int rows) { return rows * D * 2; }
};

// Rows read BOTH whole (ds_read_b128) and through ds_read_b64_tr_b16: the key permutes all chunk bits.
template <int D>
struct DualTile {
  static constexpr int CPR = D / 8;
  static constexpr int RPI = 64 / CPR;
  __host__ __device__ static constexpr int row_base(int row) { return row * D * 2; }
  // D = 128: the two 2-bit fields of row % 16 swapped (row reads need 16 rows apart in all four bits, transpose
  // reads need 4 consecutive rows apart in the upper two); D = 64: two rows per 256-byte bank cycle, so row / 2
  // (3 bits) permutes the 8 chunks, its lowest bit going to the top.
  __host__ __device__ static constexpr int key(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : (((((row >> 1) & 7) & 1) << 2) | (((row >> 1) & 7) >> 1));
  }
  __host__ __device__ static constexpr int bytes(int rows) { return rows * D * 2; }
};

// One wave-wide LDS-direct load of one dword per lane: lane L's 4 bytes land at LDS offset lds + 4 L.
__device__ inline void lds_fill_b32(i32x4 rsrc, uint32_t lds, int voff, int soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 3\n\tbuffer_load_dword %1, %2, %3 offen lds"
               :: "s"(__builtin_amdgcn_readfirstlane((int)lds)), "v"(voff), "s"(rsrc), "s"(__builtin_amdgcn_readfirstlane(soff)) : "memory");
}

// Byte offset of chunk c of row `row` inside a tile.
template <typename T>
__device__ inline int tile_off(int row, int c) { return T::row_base(row) + ((c ^ T::key(row)) << 4); }

// Per-lane part of the global offset for the LDS-direct fill of a tile by several waves: wave w fills
// tile rows rpw * w .. rpw * w + rpw - 1 with rpw / RPI instructions; in instruction i the lane
// supplies row (lane / CPR) of the RPI rows and the chunk that belongs at chunk position lane % CPR.
template <typename T>
__device__ inline int fill_voff(int rpw, int wave, int i, int lane, int row_bytes) {
  const int row = rpw * wave + T::RPI * i + lane / T::CPR;
  return row * row_bytes + (((lane % T::CPR) ^ T::key(row)) << 4);
}

// Wave-private LDS staging for writing a [32 rows x 2 D bytes] tile that the wave holds in the accumulator layout of
// the 32 x 32 matrix instructions (lane = column inside a 32-column block, register i = row reg_row(i, lane / 32)).
// Stored from that layout a wave-wide instruction carries 2 or 4 bytes per lane and the memory pipeline takes as long
// for it as for one of 16 bytes per lane, so a unit's 512 such stores cost several microseconds, which the next unit's
// first loads then queue behind.  Staged through LDS the same tile leaves in D / 16 instructions of whole rows.
// The staged row is 2 D bytes: all D channels as bf16, or D / 2 channels as fp32 (two passes).
template <int D>
struct RowStage {
  static constexpr int ROW = 2 * D + 16;           // LDS row stride: the two lane halves (4 rows apart) on different banks
  static constexpr int BYTES = 32 * ROW;
  static constexpr int CPR = D / 8;                // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;             // rows per store instruction
  static constexpr int N = 32 / RPI;
  // the staged rows are written as 2- and 4-byte values and read back as 16-byte chunks: types that may alias
  typedef uint16_t __attribute__((may_alias)) u16_any;
  typedef uint32_t __attribute__((may_alias)) u32_any;
  typedef u32x4 __attribute__((may_alias)) u32x4_any;
  __device__ static int reg_row(int i, int g2) { return 8 * (i / 4) + 4 * g2 + (i % 4); }
  __device__ static int at(int row, int byte) { return row * ROW + byte; }
  __device__ static void put_bf16(unsigned char* buf, int row, int col, float v) {
    *reinterpret_cast<u16_any*>(buf + at(row, 2 * col)) = __builtin_bit_cast(uint16_t, (__bf16)v);
  }
  __device__ static void put_f32(unsigned char* buf, int row, int col, float v) {
    *reinterpret_cast<u32_any*>(buf + at(row, 4 * col)) = __builtin_bit_cast(uint32_t, v);
  }
  // after the wave has written its staged rows: row r goes to byte offset r * row_bytes + soff0 of the resource
  // (rows past the resource's range are dropped)
  __device__ static void flush(const unsigned char* buf, int lane, __amdgpu_buffer_rsrc_t r, int row_bytes, int soff0) {
    // the lane's addresses are formed here, after the unit's loop: values that the compiler can form ahead of the loop
    // would hold registers across it
    asm volatile("" : "+v"(lane));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int row = lane / CPR, chunk = lane % CPR;
    const int voff = row * row_bytes + 16 * chunk + soff0;
    u32x4 x[N];                                    // all chunks first: one LDS latency, not N
#pragma unroll
    for (int j = 0; j < N; ++j) x[j] = *reinterpret_cast<const u32x4_any*>(buf + at(RPI * j + row, 16 * chunk));
#pragma unroll
    for (int j = 0; j < N; ++j) {
      __builtin_amdgcn_raw_buffer_store_b128(x[j], r, voff + RPI * j * row_bytes, 0, 0);
      // The data registers stay untouched for two more cycles: a 16-byte store followed at once by a vector
      // instruction that overwrites its first data register has stored the new value now and then (seen with the
      // row term in the scalar offset; the whole offset is per lane here, the case for which the compiler knows the
      // hazard, and the wait below does not depend on its table).
      asm volatile("s_nop 1" :: "v"(x[j]));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
};

// Unit queue of a persistent block.  Units are numbered per XCD counter; unit u of an XCD is
// (tile u / per_tile, sub-index u % per_tile).  Wave 0 keeps the atomic for the unit after next
// and the 64-byte record of the next unit in flight while the block computes the current one,
// so neither the atomic's nor the record's latency is paid between units.  LDS: s_next (1 word),
// s_rec (16 words).  Every thread of the block calls every function.
struct UnitQueue {
  int32_t pend, recw, idx1;
  int32_t* counter;
  const int32_t* rec_words;
  int32_t n_units, per_tile;

  __device__ void init(SchedHeader* hdr, const Tile* tiles, int xcd, int per_tile_, int32_t* s_next, int32_t* s_rec) {
    counter = &hdr->counter[xcd];
    rec_words = reinterpret_cast<const int32_t*>(tiles);
    per_tile = per_tile_;
    n_units = hdr->n_tiles * per_tile_;
    pend = recw = idx1 = 0;
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < 64) {
      int32_t v0 = 0;
      if (lane == 0) v0 = atomicAdd(counter, 1);
      const int32_t u0 = __builtin_amdgcn_readfirstlane(v0);
      if (lane == 0) pend = atomicAdd(counter, 1);
      if (lane < 16) s_rec[lane] = u0 < n_units ? rec_words[(u0 / per_tile) * 16 + lane] : 0;
      if (lane == 0) *s_next = u0;
    }
    __syncthreads();
  }
  // current unit number (>= n_units: the list is exhausted); wave-uniform
  __device__ int32_t current(const int32_t* s_next) const { return __builtin_amdgcn_readfirstlane(*s_next); }
  // after the record has been read from s_rec: start the trips for the next two units
  __device__ void prefetch() {
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x & 63;
      idx1 = __builtin_amdgcn_readfirstlane(pend);
      if (lane == 0) pend = atomicAdd(counter, 1);
      recw = (lane < 16 && idx1 < n_units) ? rec_words[(idx1 / per_tile) * 16 + lane] : 0;
    }
  }
  // end of the unit: publish the next unit to the block
  __device__ void advance(int32_t* s_next, int32_t* s_rec) {
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x & 63;
      if (lane < 16) s_rec[lane] = recw;
      if (lane == 0) *s_next = idx1;
    }
    // LDS-only barrier: the unit's last stores and atomics to global memory stay in flight (a __syncthreads() would
    // wait for them here, several microseconds per unit); nothing in the block reads them back.
    __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  }
};

// The first NW words of the unit's record (the rest of T reads as zero), as wave-uniform values.
template <typename T, int NW>
__device__ inline T read_record(const int32_t* s_rec) {
  static_assert(sizeof(T) == 64 && NW <= 16, "16-word record");
  T t;
  int32_t* tw = reinterpret_cast<int32_t*>(&t);
#pragma unroll
  for (int i = 0; i < NW; ++i) tw[i] = __builtin_amdgcn_readfirstlane(s_rec[i]);
#pragma unroll
  for (int i = NW; i < 16; ++i) tw[i] = 0;
  return t;
}

}  // namespace fcp
