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

__device__ inline f32x16 zero16() {
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  return z;
}

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
    __syncthreads();
  }
};

template <typename T>
__device__ inline T read_record(const int32_t* s_rec) {
  static_assert(sizeof(T) == 64, "16-word record");
  T t;
  int32_t* tw = reinterpret_cast<int32_t*>(&t);
#pragma unroll
  for (int i = 0; i < 12; ++i) tw[i] = __builtin_amdgcn_readfirstlane(s_rec[i]);
#pragma unroll
  for (int i = 12; i < 16; ++i) tw[i] = 0;
  return t;
}

}  // namespace fcp
